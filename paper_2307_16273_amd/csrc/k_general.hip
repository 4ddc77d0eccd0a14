// The batched matrix product proved from the three stacks themselves, in the general aggregated
// form (Sec. 4, Eq. tensor-op-aggr and Eq. tensor-op-compressed with f(a, b) = a b; Protocol
// tensor-op-aggr):
//   0 = sum_n sum_i sum_j beta~(w, n) beta~(u, i) (D2^-1 Y(n, i) - X0(n, i0, j) X1(n, j, i1)),
// i = (i0, i1) the output index, j the inner index, w and u drawn by the verifier.
//
// No table of the product size N D1 D3 D2 is ever built.  Every round polynomial separates:
//  * stack rounds:  f_t(x) = sum_n' beta~(w_[t+1:], n') (Ty_x(n') - sum_j T0_x(n', j) T1_x(n', j)) on
//    the collapsed tables Ty = Y~(., u), T0 = X0~(., u0, .), T1 = X1~(., ., u1) (the sums over i
//    against beta~(u, .) are taken once, before the rounds);
//  * rounds over i0:  g(x) = sum_b P_x(b) D_x(b) with P = beta~(u0, .) and
//    D(i0) = Y~(v_n, i0, u1) - sum_j X0~(v_n, i0, j) X1~(v_n, j, u1);
//  * rounds over i1:  the same with P = beta~(u0, v_i0) beta~(u1, .) and
//    D(i1) = Y~(v_n, v_i0, i1) - sum_j X0~(v_n, v_i0, j) X1~(v_n, j, i1);
//  * rounds over j (round r):  g(x) = c (2^-(r+1) Y~(v_n, v_i) - sum_b A_x(b) B_x(b)) with
//    c = beta~(u, v_i), A = X0~(v_n, v_i0, .), B = X1~(v_n, ., v_i1).
// The contractions between the phases are beta-weighted axis contractions of the stacks and of
// small tables; the rounds after the stack rounds run in one block per phase.
#include "dev_common.cuh"

static unsigned ga_grid(uint64_t n, unsigned cap) {
    uint64_t b = (n + ZK_BLOCK - 1) / ZK_BLOCK;
    if (b < 1) b = 1;
    return (unsigned)(b < cap ? b : cap);
}

// ---- stack rounds ------------------------------------------------------------------------------

// part[3 blk + x] = sum over this block's (n', j) of ws[n'] T0_x(n', j) T1_x(n', j), x = 0, 1, 2;
// T_x = lo + x (hi - lo) with lo = row n', hi = row n' + half
__global__ __launch_bounds__(ZK_BLOCK) void k_ga_stack_round(FrTab t0, FrTab t1, FrTab ws, uint64_t half,
                                                             uint64_t d2, Fr* part) {
    __shared__ uint32_t red[64];
    const uint64_t n = half * d2;
    Fr acc0 = fr_zero(), acc1 = fr_zero(), acc2 = fr_zero();
    for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < n; e += (uint64_t)gridDim.x * blockDim.x) {
        const Fr w = tab_ld(ws, e / d2);
        const Fr a_lo = fr_mul_ni(w, tab_ld(t0, e)), a_hi = fr_mul_ni(w, tab_ld(t0, e + n));
        const Fr b_lo = tab_ld(t1, e), b_hi = tab_ld(t1, e + n);
        acc0 = fr_add(acc0, fr_mul_ni(a_lo, b_lo));
        acc1 = fr_add(acc1, fr_mul_ni(a_hi, b_hi));
        acc2 = fr_add(acc2, fr_mul_ni(fr_sub(fr_dbl(a_hi), a_lo), fr_sub(fr_dbl(b_hi), b_lo)));
    }
    acc0 = block_sum(acc0, red);
    acc1 = block_sum(acc1, red);
    acc2 = block_sum(acc2, red);
    if (threadIdx.x == 0) {
        part[3 * blockIdx.x + 0] = acc0;
        part[3 * blockIdx.x + 1] = acc1;
        part[3 * blockIdx.x + 2] = acc2;
    }
}

struct GaStackFinArgs {
    DevState* st;
    const Fr* part;
    int nblk;
    FrTab ty, ws;
    uint64_t half;
    uint32_t proof_off;
    int chal_idx;
};

// f_t(0), f_t(1), f_t(2) -> proof and transcript ("f", all three), v_t drawn, claim = f_t(v_t),
// Ty folded with v_t
__global__ __launch_bounds__(ZK_BLOCK) void k_ga_stack_finalise(GaStackFinArgs a) {
    __shared__ TsShared S;
    __shared__ Fr g[4];
    __shared__ uint32_t red[64];
    DevState* st = a.st;
    block_ts_load(S, st);
    block_reduce_partials(a.part, a.nblk, 3, g);
    Fr y0 = fr_zero(), y1 = fr_zero();
    for (uint64_t n = threadIdx.x; n < a.half; n += blockDim.x) {
        const Fr w = tab_ld(a.ws, n);
        y0 = fr_add(y0, fr_mul_ni(w, tab_ld(a.ty, n)));
        y1 = fr_add(y1, fr_mul_ni(w, tab_ld(a.ty, n + a.half)));
    }
    y0 = block_sum(y0, red);
    y1 = block_sum(y1, red);
    if (threadIdx.x == 0) {
        g[0] = fr_sub(y0, g[0]);
        g[1] = fr_sub(y1, g[1]);
        g[2] = fr_sub(fr_sub(fr_dbl(y1), y0), g[2]);
    }
    __syncthreads();
    const Fr v = block_round_challenge(S, st, g, 3, a.proof_off, a.chal_idx, 'f', false);
    if ((threadIdx.x >> 6) == 1) {
        const Fr c = wave_lagrange(S.tmp, 3, v);
        if ((threadIdx.x & 63) == 0) {
            st->claim = c;
            st->lag_npts = 0;
        }
    }
    for (uint64_t n = threadIdx.x; n < a.half; n += blockDim.x) {
        const Fr lo = tab_ld(a.ty, n), hi = tab_ld(a.ty, n + a.half);
        tab_st(a.ty, n, fr_add(lo, fr_mul_ni(v, fr_sub(hi, lo))));
    }
    block_ts_store(S, st);
}

// t[e] <- t[e] + v (t[e + n] - t[e]), e < n, for both tables; v = chal[chal_idx]
__global__ __launch_bounds__(ZK_BLOCK) void k_ga_fold2(const DevState* st, int chal_idx, FrTab t0, FrTab t1,
                                                       uint64_t n) {
    const Fr v = st->chal[chal_idx];
    for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < n; e += (uint64_t)gridDim.x * blockDim.x) {
        const Fr a_lo = tab_ld(t0, e), a_hi = tab_ld(t0, e + n);
        tab_st(t0, e, fr_add(a_lo, fr_mul_ni(v, fr_sub(a_hi, a_lo))));
        const Fr b_lo = tab_ld(t1, e), b_hi = tab_ld(t1, e + n);
        tab_st(t1, e, fr_add(b_lo, fr_mul_ni(v, fr_sub(b_hi, b_lo))));
    }
}

// ---- rounds over i0, i1, j: one block per phase --------------------------------------------------

struct GaInnerArgs {
    DevState* st;
    FrTab p;           // modes 1, 2: the weights (folded in place); mode 3: A
    FrTab q;           // modes 1, 2: the Y side (read only); mode 3: B
    FrTab z;           // modes 1, 2: the product side, turned into D = q - z in place; mode 3: one entry, Y~(v_n, v_i)
    int mode;          // 1: i0, 2: i1, 3: j
    int rounds;        // log2 of the table length
    int chal_base;     // challenge index of the phase's first round
    uint32_t rounds_off;
    uint32_t claim_off;    // mode 1: claim_0 of the SC block
    uint32_t finals_off;   // mode 3
    int zero_claim;        // mode 1 without stack rounds: the claim is 0
    int scal_c;            // scal slot of beta~(u0, v_i0) (mode 1 writes, 2 reads) / beta~(u, v_i) (2 writes, 3 reads)
    int scal_fin;          // mode 3: finals Y~, X0~, X1~ -> scal[scal_fin ..)
};

__global__ __launch_bounds__(ZK_BLOCK) void k_ga_inner(GaInnerArgs a) {
    __shared__ TsShared S;
    __shared__ Fr g[4];
    __shared__ uint32_t red[64];
    DevState* st = a.st;
    const int tid = threadIdx.x;
    block_ts_load(S, st);
    const uint64_t len = (uint64_t)1 << a.rounds;
    if (a.mode != 3) {
        const Fr c0 = a.mode == 2 ? st->scal[a.scal_c] : fr_one();
        for (uint64_t b = tid; b < len; b += blockDim.x) {
            tab_st(a.z, b, fr_sub(tab_ld(a.q, b), tab_ld(a.z, b)));
            if (a.mode == 2) tab_st(a.p, b, fr_mul_ni(c0, tab_ld(a.p, b)));
        }
    }
    if (a.mode == 1 && tid == 0) {
        // claim_0 = f_{n-1}(v_{n-1}), or 0 without stack rounds: fixed by the transcript, written only
        if (a.zero_claim) st->claim = fr_zero();
        const Fr plain = fr_from_mont_ni(a.zero_claim ? fr_zero() : st->claim);
        uint32_t* dst = (uint32_t*)(st->proof + a.claim_off);
#pragma unroll
        for (int l = 0; l < 8; ++l) dst[l] = plain.v[l];
    }
    __syncthreads();
    const Fr c = a.mode == 3 ? st->scal[a.scal_c] : fr_zero();
    const Fr yf = a.mode == 3 ? tab_ld(a.z, 0) : fr_zero();
    Fr ky = yf;   // mode 3: 2^-r Y~ before round r
    const FrTab d = a.mode == 3 ? a.q : a.z;   // the table next to p in the rounds
    for (int r = 0; r < a.rounds; ++r) {
        const uint64_t m = len >> (r + 1);
        Fr acc0 = fr_zero(), acc1 = fr_zero(), acc2 = fr_zero();
        for (uint64_t b = tid; b < m; b += blockDim.x) {
            const Fr p_lo = tab_ld(a.p, b), p_hi = tab_ld(a.p, b + m);
            const Fr q_lo = tab_ld(d, b), q_hi = tab_ld(d, b + m);
            acc0 = fr_add(acc0, fr_mul_ni(p_lo, q_lo));
            acc1 = fr_add(acc1, fr_mul_ni(p_hi, q_hi));
            acc2 = fr_add(acc2, fr_mul_ni(fr_sub(fr_dbl(p_hi), p_lo), fr_sub(fr_dbl(q_hi), q_lo)));
        }
        acc0 = block_sum(acc0, red);
        acc1 = block_sum(acc1, red);
        acc2 = block_sum(acc2, red);
        if (a.mode == 3) ky = fr_mul_ni(ky, st->inv2);
        if (tid == 0) {
            if (a.mode == 3) {
                g[0] = fr_mul_ni(c, fr_sub(ky, acc0));
                g[1] = fr_mul_ni(c, fr_sub(ky, acc1));
                g[2] = fr_mul_ni(c, fr_sub(ky, acc2));
            } else {
                g[0] = acc0;
                g[1] = acc1;
                g[2] = acc2;
            }
        }
        __syncthreads();
        const Fr v = block_finalise_round(S, st, g, 3, a.rounds_off + 96u * (uint32_t)r, a.chal_base + r);
        for (uint64_t b = tid; b < m; b += blockDim.x) {
            const Fr p_lo = tab_ld(a.p, b), p_hi = tab_ld(a.p, b + m);
            tab_st(a.p, b, fr_add(p_lo, fr_mul_ni(v, fr_sub(p_hi, p_lo))));
            const Fr q_lo = tab_ld(d, b), q_hi = tab_ld(d, b + m);
            tab_st(d, b, fr_add(q_lo, fr_mul_ni(v, fr_sub(q_hi, q_lo))));
        }
        __syncthreads();
    }
    if (a.mode != 3) {
        if (tid == 0) st->scal[a.scal_c] = tab_ld(a.p, 0);
    } else {
        if (tid == 0) {
            g[0] = yf;
            g[1] = tab_ld(a.p, 0);
            g[2] = tab_ld(d, 0);
            for (int k = 0; k < 3; ++k) st->scal[a.scal_fin + k] = g[k];
        }
        __syncthreads();
        block_absorb_frs(S, 'f', g, 3, (uint32_t*)(st->proof + a.finals_off));
    }
    block_ts_store(S, st);
}

// ---- host side ---------------------------------------------------------------------------------

static const void* ga_src(const zkdl_tensor* X, FrTab* holder) {
    *holder = make_tab(X->data, X->numel);
    return X->kind == TK_FR ? (const void*)holder : X->data;
}

// X0 [N, D1, D2], X1 [N, D2, D3], Y [N, D1, D3] (all extents powers of two, checked by the caller).
// Header frame, the draw of (w, u), the "ZKGA" block; finals Y~, X0~, X1~ -> scal[scal_base ..).
int zk_matmul_general(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1, const zkdl_tensor* Y, int ln,
                      int l1, int l2, int l3, int scal_base) {
    const uint64_t N = (uint64_t)1 << ln, D1 = (uint64_t)1 << l1, D2 = (uint64_t)1 << l2, D3 = (uint64_t)1 << l3;
    const int n_inner = l1 + l3 + l2;
    if (ln > 13 || ctx->n_chal + 2 * ln + 2 * (l1 + l3) + l2 > ZK_MAX_CHAL) return ZKDL_EINVAL;
    uint32_t hdr[4] = {(uint32_t)N, (uint32_t)D1, (uint32_t)D2, (uint32_t)D3};
    zk_absorb_words(ctx, "tensor_op_aggr", hdr, 4);
    const int cw = ctx->n_chal, cu0 = cw + ln, cu1 = cu0 + l1;
    zk_launch_draw(ctx, cw, ln + l1 + l3);
    ctx->n_chal += ln + l1 + l3;
    const int cvn = ctx->n_chal, cvi0 = cvn + ln, cvi1 = cvi0 + l1, cvj = cvi1 + l3;
    ctx->n_chal += ln + n_inner;
    const Fr* chal = ctx->dev->chal;

    uint32_t phdr[8] = {0x41474B5Au, (uint32_t)ln, (uint32_t)l1, (uint32_t)l3, (uint32_t)l2, 0, 0, 0};
    zk_write_proof_words(ctx, phdr, 8);
    const uint32_t stack_off = (uint32_t)ctx->proof_len;
    ctx->proof_len = stack_off + 96 * (size_t)ln;
    uint32_t ihdr[4] = {0x43534B5Au, 3, 2, (uint32_t)n_inner};
    zk_write_proof_words(ctx, ihdr, 4);
    const uint32_t claim_off = (uint32_t)ctx->proof_len;
    const uint32_t rounds_off = claim_off + 32;
    const uint32_t finals_off = rounds_off + 96 * (uint32_t)n_inner;
    if ((size_t)finals_off + 96 > (size_t)ZK_PROOF_CAP) return ZKDL_ESMALL;
    ctx->proof_len = finals_off + 96;

    const uint64_t elems = 3 * N + 4 * D1 + 4 * D3 + 2 * D2 + N * D3 + 2 * N * D2 + D1 * D3 + D1 * D2 + D2 * D3 +
                           D1 + D3 + D2 + 8;
    void* mem = zk_alloc(ctx, elems * 32);
    if (!mem) return ZKDL_ENOMEM;
    uint32_t* cur = (uint32_t*)mem;
    auto take = [&](uint64_t n) {
        FrTab t = make_tab(cur, n);
        cur += 8 * n;
        return t;
    };
    FrTab wsuf[16];
    BetaJob jobs[16];
    int nj = 0;
    for (int t = 0; t < ln; ++t) {
        wsuf[t] = take((uint64_t)1 << (ln - t - 1));
        jobs[nj++] = BetaJob{chal + cw + t + 1, ln - t - 1, wsuf[t]};
    }
    FrTab bu0 = take(D1), bu1 = take(D3);
    jobs[nj++] = BetaJob{chal + cu0, l1, bu0};
    jobs[nj++] = BetaJob{chal + cu1, l3, bu1};
    FrTab ty = take(N), ty_mid = take(N * D3), t0u = take(N * D2), t1u = take(N * D2);
    FrTab bvn = take(N), yv = take(D1 * D3), x0v = take(D1 * D2), x1v = take(D2 * D3);
    FrTab yc = take(D1), z0 = take(D1), bvi0 = take(D1);
    FrTab yr = take(D3), x0r = take(D2), z1 = take(D3), bvi1 = take(D3);
    FrTab bj = take(D2), yf = take(1);

    FrTab h0, h1, hy;
    const void* s0 = ga_src(X0, &h0);
    const void* s1 = ga_src(X1, &h1);
    const void* sy = ga_src(Y, &hy);
    int rc = zk_build_beta_many(ctx, jobs, nj);
    // the sums over the output index against beta~(u, .)
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, Y->kind, sy, N, D1, D3, bu0, ty_mid);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_FR, &ty_mid, N, D3, 1, bu1, ty);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, X0->kind, s0, N, D1, D2, bu0, t0u);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, X1->kind, s1, N * D2, D3, 1, bu1, t1u);
    if (rc != ZKDL_OK) {
        zk_free(ctx, mem);
        return rc;
    }
    for (int t = 0; t < ln; ++t) {
        const uint64_t half = (uint64_t)1 << (ln - t - 1);
        const unsigned grid = ga_grid(half * D2, ZK_MAX_PART_BLOCKS);
        zk_prof_begin(ctx, ZKDL_PROF_SC_ROUND_FIRST, 128.0 * (double)(half * D2));
        hipLaunchKernelGGL(k_ga_stack_round, dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, t0u, t1u, wsuf[t], half, D2,
                           ctx->partials);
        zk_prof_end(ctx);
        GaStackFinArgs fa;
        fa.st = ctx->dev;
        fa.part = ctx->partials;
        fa.nblk = (int)grid;
        fa.ty = ty;
        fa.ws = wsuf[t];
        fa.half = half;
        fa.proof_off = stack_off + 96u * (uint32_t)t;
        fa.chal_idx = cvn + t;
        zk_prof_begin(ctx, ZKDL_PROF_FINALISE, 96.0);
        hipLaunchKernelGGL(k_ga_stack_finalise, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, fa);
        zk_prof_end(ctx);
        hipLaunchKernelGGL(k_ga_fold2, dim3(ga_grid(half * D2, 4096)), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev,
                           cvn + t, t0u, t1u, half * D2);
    }
    // the stacks at v_n; t0u, t1u now hold X0~(v_n, u0, .) and X1~(v_n, ., u1) in their first D2 entries
    rc = zk_build_beta(ctx, chal + cvn, ln, bvn);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, Y->kind, sy, 1, N, D1 * D3, bvn, yv);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, X0->kind, s0, 1, N, D1 * D2, bvn, x0v);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, X1->kind, s1, 1, N, D2 * D3, bvn, x1v);
    // rounds over i0
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_FR, &yv, D1, D3, 1, bu1, yc);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_FR, &x0v, D1, D2, 1, t1u, z0);
    GaInnerArgs ia;
    ia.st = ctx->dev;
    ia.scal_c = scal_base + 3;
    ia.scal_fin = scal_base;
    ia.claim_off = claim_off;
    ia.finals_off = finals_off;
    ia.zero_claim = ln == 0;
    if (rc == ZKDL_OK) {
        ia.p = bu0;
        ia.q = yc;
        ia.z = z0;
        ia.mode = 1;
        ia.rounds = l1;
        ia.chal_base = cvi0;
        ia.rounds_off = rounds_off;
        hipLaunchKernelGGL(k_ga_inner, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ia);
    }
    // rounds over i1
    if (rc == ZKDL_OK) rc = zk_build_beta(ctx, chal + cvi0, l1, bvi0);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_FR, &yv, 1, D1, D3, bvi0, yr);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_FR, &x0v, 1, D1, D2, bvi0, x0r);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_FR, &x1v, 1, D2, D3, x0r, z1);
    if (rc == ZKDL_OK) {
        ia.p = bu1;
        ia.q = yr;
        ia.z = z1;
        ia.mode = 2;
        ia.rounds = l3;
        ia.chal_base = cvi1;
        ia.rounds_off = rounds_off + 96u * (uint32_t)l1;
        hipLaunchKernelGGL(k_ga_inner, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ia);
    }
    // rounds over j
    if (rc == ZKDL_OK) rc = zk_build_beta(ctx, chal + cvi1, l3, bvi1);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_FR, &x1v, D2, D3, 1, bvi1, bj);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_FR, &yr, 1, D3, 1, bvi1, yf);
    if (rc == ZKDL_OK) {
        ia.p = x0r;
        ia.q = bj;
        ia.z = yf;
        ia.mode = 3;
        ia.rounds = l2;
        ia.chal_base = cvj;
        ia.rounds_off = rounds_off + 96u * (uint32_t)(l1 + l3);
        hipLaunchKernelGGL(k_ga_inner, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ia);
    }
    zk_free(ctx, mem);
    return rc;
}
