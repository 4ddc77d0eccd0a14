// zkReLU (Sec. 3.1, App. A): the combined sumcheck of the six equations
//   forward in / out / binarity, backward in / out / binarity
// with weights r^2, r, 1, r'r^2, r'r, r', over aux in {0,1}^{2 x D x J}
// (J = Q+R padded to a power of two), followed by the merge of the three claims
// on aux into one.
//
// How the sum is organised here (same field elements as the direct double sum
// over (i, j), grouped differently):
//  * The "in" and "out" equations are linear in aux along j, and
//    sum_j aux(k,i,j) s(j) is the integer itself (Eqs. aux-Z, aux-GA) while
//    sum_j aux(k,i,j) s'(j) is the rescaled integer.  Folding over i commutes with
//    these sums, so during the i-rounds they run on D-sized tables
//    (lin_body): beta*Z, beta*(1-sign)*Z', beta*G_A, beta*(1-sign)*G_A'.
//  * Only the binarity terms need the D x (Q+R) tables (bin*_body).  Their
//    equality factor splits as beta~(u_bin,(i,j)) = beta_I(i) beta_J(j).
//    Rounds 0 to 3 work on the integers directly: aux is binary, so in round 0
//    a(x)^2 - a(x) = (x^2 - x) [bit_lo != bit_hi]; with t challenges bound an entry is a
//    combination of 2^t bits whose coefficients add up to one, which makes round 1 a
//    quadratic form in the bits: masked sums of beta_J and five products (bin1_body);
//    rounds 2 and 3 read an entry's value from a 16- / 256-entry table by its bits
//    (bin2_body, bin3_body).  After the fourth challenge the columns are written out
//    once (k_zk_mat4), column-major: entry (k, j, i) at plane (k*(Q+R)+j), so
//    that threads over i read coalesced limb planes; D/16 rows.  Later rounds fold them
//    (binp_body, binl_body).  Sums over j of beta_J(j) (...) are accumulated as 64-bit columns
//    and reduced once per pair index.  From round 1 on a round leaves its column sums
//    SA, SC, SD per pair index for the next one (psum_bind), which then squares only
//    hi - lo per column.  beta_I is folded by the binarity blocks themselves between
//    two buffers, so they share no table with the linear blocks.
//  * The first two rounds of the linear equations and the input claims read the integers
//    (9 x 2 limb products, no value tables before round 1: lin0_int_body, lin1_int_body,
//    k_zk_prepare_int) and take the equality tables over i as products of two factors of
//    about sqrt(D) entries (SplitEq); round 1 writes all folded tables for the later rounds.
//  * One launch per i-round (k_zk_round): the first blocks take the linear equations,
//    the others the binarity terms; the round's finaliser adds up all partial sums.
//    Rounds with few pairs spread a pair over more threads (lin_body_small, column
//    and slice chunks) so that no thread carries a long chain of products.
//  * The j-rounds (log2 J of them) and the merge run on 64/128-entry tables in a
//    single block (k_zk_tail) together with their transcript steps.
#include "dev_common.cuh"

namespace {

constexpr int LIN_TABLES = 10;
// order of the D-sized tables
enum { T_BZ = 0, T_Z, T_BA, T_NS, T_ZP, T_BGA, T_GA, T_BGZ, T_GAP, T_BI };

// The D-sized tables live as lazy 29-bit limbs (nine planes): they are folded every round.
struct ZkTabs {
    F9Tab t[LIN_TABLES];
};
// the five equality tables as built (packed): beta_Z, beta_A, beta_GA, beta_GZ, beta_I
struct ZkBeta8 {
    FrTab t[5];
};

// An equality table over i in two factors: beta~(u, i) = H[i >> lb] L[i & (2^lb - 1)], H over the
// leading variables of u and L over the others.  While the variables that the rounds bind lie in
// H, the table over i is never built: an entry is one product of two entries of tables of about
// sqrt(D) elements, which stay in cache, and binding a challenge folds H alone.  The first two
// i-rounds work this way; round 1 writes the folded tables (D/2 entries) for the later rounds.
struct SplitEq {
    F9Tab H[5], L[5];   // Z, A, G_A, G_Z (times the weights of their equations once those are drawn), I
    int lb;
};

__device__ __forceinline__ F9 split_entry(const F9Tab& H, const F9Tab& L, int lb, uint64_t i) {
    // factors normal and below 2.41 r: the product is normal and below 2 r
    return f9_mul(f9tab_ld(H, i >> lb), f9tab_ld(L, i & (((uint64_t)1 << lb) - 1)));
}

struct SplitConvArgs {
    FrTab src[10];     // packed tables as built: H of the five points, then L
    F9Tab dst[10];
    uint64_t n[10];
};

// packed -> lazy limbs, table blockIdx.y
__global__ __launch_bounds__(ZK_BLOCK) void k_zk_split_convert(SplitConvArgs a) {
    const int q = blockIdx.y;
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < a.n[q]; i += (uint64_t)gridDim.x * blockDim.x)
        f9tab_st(a.dst[q], i, fr_unpack(tab_ld(a.src[q], i)));
}

// H of the four linear equations times the weight of the equation (in place), once r, r' are drawn
__global__ __launch_bounds__(ZK_BLOCK) void k_zk_split_scale(SplitEq sp, uint64_t nh, const Fr* weights, int has_ga) {
    const int e = blockIdx.y;
    if (e >= 2 && !has_ga) return;
    const F9 w = fr_unpack(weights[e]);
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < nh; i += (uint64_t)gridDim.x * blockDim.x)
        f9tab_st(sp.H[e], i, f9_cond_sub(f9_mul(f9tab_ld(sp.H[e], i), w)));
}

// binds the leading variable of the five H tables: dst[j] = src[j] + v (src[j + half] - src[j])
__global__ __launch_bounds__(ZK_BLOCK) void k_zk_split_fold(SplitEq src, SplitEq dst, uint64_t half, const Fr* v, int has_ga) {
    const int e = blockIdx.y;
    if ((e == 2 || e == 3) && !has_ga) return;
    const F9 v9 = fr_unpack(*v);
    for (uint64_t j = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; j < half; j += (uint64_t)gridDim.x * blockDim.x) {
        const F9 lo = f9tab_ld(src.H[e], j), hi = f9tab_ld(src.H[e], j + half);
        f9tab_st(dst.H[e], j, f9_norm_reduce(f9_add(lo, f9_mul(f9_sub(hi, lo), v9))));
    }
}

__device__ __forceinline__ int64_t rescale_half_up(int64_t x, int r_bits) {
    // floor((x + 2^(R-1)) / 2^R) as the recomposition Z' = aux[R:Q+R] . s_Q + aux[R-1] (Sec. 3.1) writes it:
    // the value above bit R plus bit R-1; no sum that could leave the 64-bit range (R = 1, x = INT64_MAX)
    return (x >> r_bits) + ((x >> (r_bits - 1)) & 1);
}

__device__ __forceinline__ bool in_range(int64_t x, int nbits) {
    if (nbits >= 64) return true;
    int64_t top = x >> (nbits - 1);
    return top == 0 || top == -1;
}

// ---------------------------------------------------------------------------
// prepare: the D-sized value tables and the four input claims
// ---------------------------------------------------------------------------
struct PrepArgs {
    const int64_t* z;
    const int64_t* ga;   // nullptr: G_A = 0
    uint64_t D;
    int nbits, r_bits;
    ZkBeta8 beta;        // packed equality tables, read
    ZkTabs tabs;         // value tables, written if write_vals
    int write_vals;      // 0: the first two i-rounds read the integers themselves
    SplitEq sp;          // k_zk_prepare_int: the equality tables in two factors, as built
    Fr* part;            // per block: 4 partial dot products
    DevState* st;
};

__global__ __launch_bounds__(ZK_BLOCK) void k_zk_prepare(PrepArgs a) {
    __shared__ uint32_t red[64];
    Fr acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = fr_zero();
    bool bad = false;
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < a.D;
         i += (uint64_t)gridDim.x * blockDim.x) {
        int64_t z = a.z[i];
        bad |= !in_range(z, a.nbits);
        bool neg = (z >> (a.nbits - 1)) & 1;            // aux(0, i, Q+R-1)
        int64_t zp = rescale_half_up(z, a.r_bits);
        Fr fz = fr_from_i64(z), fzp = fr_from_i64(zp);
        if (a.write_vals) {
            f9tab_st(a.tabs.t[T_Z], i, fr_unpack(fz));
            f9tab_st(a.tabs.t[T_ZP], i, fr_unpack(fzp));
            f9tab_st(a.tabs.t[T_NS], i, fr_unpack(neg ? fr_zero() : fr_one()));
        }
        acc[0] = fr_add(acc[0], fr_mul(tab_ld(a.beta.t[0], i), fz));
        if (!neg) acc[1] = fr_add(acc[1], fr_mul(tab_ld(a.beta.t[1], i), fzp));
        if (a.ga) {
            int64_t g = a.ga[i];
            bad |= !in_range(g, a.nbits);
            int64_t gp = rescale_half_up(g, a.r_bits);
            Fr fg = fr_from_i64(g), fgp = fr_from_i64(gp);
            if (a.write_vals) {
                f9tab_st(a.tabs.t[T_GA], i, fr_unpack(fg));
                f9tab_st(a.tabs.t[T_GAP], i, fr_unpack(fgp));
            }
            acc[2] = fr_add(acc[2], fr_mul(tab_ld(a.beta.t[2], i), fg));
            if (!neg) acc[3] = fr_add(acc[3], fr_mul(tab_ld(a.beta.t[3], i), fgp));
        }
    }
    if (bad) atomicOr(&a.st->err, 1u);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        Fr s = block_sum(acc[q], red);
        if (threadIdx.x == 0) a.part[(uint64_t)blockIdx.x * 4 + q] = s;
    }
}

struct ClaimsArgs {
    const Fr* part;
    int nblk;
    DevState* st;
    uint32_t claims_off;   // four input claims
    uint32_t claim0_off;   // claim_0 of the combined sumcheck
    int chal_r;            // index of r; r' follows
};

// input claims -> proof and transcript; draw r, r'; weights; combined claim
__global__ __launch_bounds__(ZK_BLOCK) void k_zk_claims(ClaimsArgs a) {
    __shared__ uint32_t red[64];
    __shared__ TsShared S;
    __shared__ Fr c[4];
    DevState* st = a.st;
    block_ts_load(S, st);
    for (int q = 0; q < 4; ++q) {
        Fr s = fr_zero();
        for (int b = threadIdx.x; b < a.nblk; b += blockDim.x) s = fr_add(s, a.part[(uint64_t)b * 4 + q]);
        s = block_sum(s, red);
        if (threadIdx.x == 0) c[q] = s;
    }
    __syncthreads();
    if (threadIdx.x < 4) st->scal[threadIdx.x] = c[threadIdx.x];
    block_absorb_frs(S, 'c', c, 4, (uint32_t*)(st->proof + a.claims_off));
    block_challenges(S, st, a.chal_r, 2);   // r, r': one draw
    block_ts_store(S, st);
    if (threadIdx.x != 0) return;
    Fr r = st->chal[a.chal_r];
    Fr rp = st->chal[a.chal_r + 1];
    Fr r2 = fr_mul_ni(r, r);
    st->weights[0] = r2;
    st->weights[1] = r;
    st->weights[2] = fr_mul_ni(rp, r2);
    st->weights[3] = fr_mul_ni(rp, r);
    st->weights[4] = rp;
    Fr claim = fr_zero();
    for (int q = 0; q < 4; ++q) claim = fr_add(claim, fr_mul_ni(st->weights[q], c[q]));
    st->claim = claim;
    st->lag_npts = 0;
    Fr plain = fr_from_mont_ni(claim);
    uint32_t* dst = (uint32_t*)(st->proof + a.claim0_off);
    for (int l = 0; l < 8; ++l) dst[l] = plain.v[l];
}

// the equation weights go into the four equality tables (beta_Z *= r^2, beta_A *= r, ...);
// all five are rewritten as lazy limbs for the rounds
__global__ __launch_bounds__(ZK_BLOCK) void k_zk_scale(ZkBeta8 beta, ZkTabs tabs, uint64_t D, const Fr* weights,
                                                       int has_ga) {
    Fr w0 = weights[0], w1 = weights[1], w2 = weights[2], w3 = weights[3];
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < D;
         i += (uint64_t)gridDim.x * blockDim.x) {
        f9tab_st(tabs.t[T_BZ], i, fr_unpack(fr_mul(tab_ld(beta.t[0], i), w0)));
        f9tab_st(tabs.t[T_BA], i, fr_unpack(fr_mul(tab_ld(beta.t[1], i), w1)));
        if (has_ga) {
            f9tab_st(tabs.t[T_BGA], i, fr_unpack(fr_mul(tab_ld(beta.t[2], i), w2)));
            f9tab_st(tabs.t[T_BGZ], i, fr_unpack(fr_mul(tab_ld(beta.t[3], i), w3)));
        }
        f9tab_st(tabs.t[T_BI], i, fr_unpack(tab_ld(beta.t[4], i)));
    }
}

// ---------------------------------------------------------------------------
// i-rounds, linear equations on the D-sized tables
// ---------------------------------------------------------------------------
struct LinArgs {
    ZkTabs tabs;
    uint64_t m;
    const Fr* chal;
    Fr* part;
    int has_ga;
    // rounds 0 and 1 on the integers (from_ints): the value tables Z, Z', 1 - sign, G_A, G_A' do
    // not exist yet; round 1 writes them, folded, for the later rounds
    int from_ints;
    const int64_t* z;
    const int64_t* ga;
    int nbits, r_bits;
    SplitEq sp;            // with from_ints: the equality tables in two factors (H bound as far as the round needs)
    unsigned eq_blocks;    // round 0 with from_ints: blocks per equation (block / eq_blocks = equation)
    int split_eq;          // the equality tables of this round come from sp (rounds >= 2 as well, value tables in memory)
    int write_eq;          // ... and are written out folded for the next round, which reads them from memory
};

// pair (lo, hi) of a lazy table, folded with the previous challenge first when FOLD; both
// normal with value < 2.41 r (the invariants of the product round kernel apply)
template <bool FOLD>
__device__ __forceinline__ void lin_pair(const F9Tab& t, uint64_t b, uint64_t m, const F9& v, F9& lo, F9& hi) {
    if (FOLD) {
        const F9 t0 = f9tab_ld(t, b), t1 = f9tab_ld(t, b + m), t2 = f9tab_ld(t, b + 2 * m), t3 = f9tab_ld(t, b + 3 * m);
        lo = f9_norm_reduce(f9_add(t0, f9_mul(f9_sub(t2, t0), v)));
        hi = f9_norm_reduce(f9_add(t1, f9_mul(f9_sub(t3, t1), v)));
        f9tab_st(t, b, lo);
        f9tab_st(t, b + m, hi);
    } else {
        lo = f9tab_ld(t, b);
        hi = f9tab_ld(t, b + m);
    }
}

// pair (lo, hi) of the equality table of equation e (table `tab` when it lives in memory): from the two
// factors while the round's variable lies in H (SPLIT), written out only when the next round reads it
// from memory
template <bool FOLD, bool SPLIT>
__device__ __forceinline__ void eq_pair(const LinArgs& a, int e, int tab, uint64_t b, uint64_t m, const F9& v, F9& lo, F9& hi) {
    if (SPLIT) {
        lo = split_entry(a.sp.H[e], a.sp.L[e], a.sp.lb, b);
        hi = split_entry(a.sp.H[e], a.sp.L[e], a.sp.lb, b + m);
        if (a.write_eq) {
            f9tab_st(a.tabs.t[tab], b, lo);
            f9tab_st(a.tabs.t[tab], b + m, hi);
        }
    } else {
        lin_pair<FOLD>(a.tabs.t[tab], b, m, v, lo, hi);
    }
}

// lo + x (hi - lo) at x = 0, 2, 3; NORMAL: all three normal, else limbs below 2^30.6
template <bool NORMAL>
__device__ __forceinline__ void line3(const F9& lo, const F9& hi, F9 e[3]) {
    const F9 dn = f9_norm(f9_sub(hi, lo));
    e[0] = lo;
    e[1] = f9_add(hi, dn);
    e[2] = f9_add(e[1], dn);
    if (NORMAL) {
        e[1] = f9_norm(e[1]);
        e[2] = f9_norm(e[2]);
    }
}

// Linear equations of one i-round: sum over i' of
//   (r^2 beta_Z) Z + (r beta_A)(1 - sign) Z' + (r'r^2 beta_GA) G_A + (r'r beta_GZ)(1 - sign) G_A'
// at x = 0, 2, 3 (x = 1 comes from the claim).
template <bool FOLD, bool SPLIT>
__device__ __forceinline__ void lin_body(const LinArgs& a, const unsigned bx, const unsigned gx) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    F9 acc[3];
#pragma unroll
    for (int x = 0; x < 3; ++x) acc[x] = f9_zero();
    F9 v = f9_zero();
    if (FOLD) v = fr_unpack(*a.chal);
    const uint64_t m = a.m;
    for (uint64_t b = bx * (uint64_t)blockDim.x + threadIdx.x; b < m;
         b += (uint64_t)gx * blockDim.x) {
        F9 lo, hi, ns[3], p[3], q[3];
        lin_pair<FOLD>(a.tabs.t[T_NS], b, m, v, lo, hi);
        line3<false>(lo, hi, ns);
        eq_pair<FOLD, SPLIT>(a, 0, T_BZ, b, m, v, lo, hi);
        line3<true>(lo, hi, p);
        lin_pair<FOLD>(a.tabs.t[T_Z], b, m, v, lo, hi);
        line3<false>(lo, hi, q);
#pragma unroll
        for (int x = 0; x < 3; ++x) acc[x] = f9_add(acc[x], f9_mul(p[x], q[x]));
        eq_pair<FOLD, SPLIT>(a, 1, T_BA, b, m, v, lo, hi);
        line3<true>(lo, hi, p);
        lin_pair<FOLD>(a.tabs.t[T_ZP], b, m, v, lo, hi);
        line3<false>(lo, hi, q);
#pragma unroll
        for (int x = 0; x < 3; ++x) acc[x] = f9_add(acc[x], f9_mul(f9_mul(p[x], ns[x]), q[x]));
#pragma unroll
        for (int x = 0; x < 3; ++x) acc[x] = f9_norm_reduce(acc[x]);
        if (a.has_ga) {
            eq_pair<FOLD, SPLIT>(a, 2, T_BGA, b, m, v, lo, hi);
            line3<true>(lo, hi, p);
            lin_pair<FOLD>(a.tabs.t[T_GA], b, m, v, lo, hi);
            line3<false>(lo, hi, q);
#pragma unroll
            for (int x = 0; x < 3; ++x) acc[x] = f9_add(acc[x], f9_mul(p[x], q[x]));
            eq_pair<FOLD, SPLIT>(a, 3, T_BGZ, b, m, v, lo, hi);
            line3<true>(lo, hi, p);
            lin_pair<FOLD>(a.tabs.t[T_GAP], b, m, v, lo, hi);
            line3<false>(lo, hi, q);
#pragma unroll
            for (int x = 0; x < 3; ++x) acc[x] = f9_add(acc[x], f9_mul(f9_mul(p[x], ns[x]), q[x]));
#pragma unroll
            for (int x = 0; x < 3; ++x) acc[x] = f9_norm_reduce(acc[x]);
        }
    }
    {   // thread j holds the sum for x = 0, 2, 3; g(1) is derived from the claim
        const Fr s = block_sum_lazy<3>(acc, red);
        Fr* pp = a.part + (uint64_t)bx * 4;
        if (threadIdx.x < 3) pp[threadIdx.x ? threadIdx.x + 1 : 0] = s;
        else if (threadIdx.x == 3) pp[1] = fr_zero();
    }
}

// ---- rounds 0 and 1 of the linear equations on the integers --------------------------------
// The value tables hold integers of at most 56 bits (Z, G_A), their rescaled values and the bit
// 1 - sign.  A table entry in Montgomery form times a plain integer is the Montgomery form of the
// product, so in round 0 a term  (weight beta)(x) * value(x)  is a 9-limb by 2-limb product with no
// reduction: the lines of the value tables through x = 0, 2, 3 are integers below 2^58 in
// magnitude.  The products are accumulated as 64-bit columns (11 of them) and reduced once per
// thread.  Round 1 binds v0 on the way: a + v0 (a' - a) for integers a, a' is
// redc(R^2 |a| +- v0 R^2 |a' - a|), one reduction and no full product; the folded tables are written
// out for the later rounds, which work on field elements as before.

// lo + x (hi - lo) at x = 0, 2, 3, each normal and below 2.41 r
__device__ __forceinline__ void line3_reduced(const F9& lo, const F9& hi, F9 e[3]) {
    const F9 dn = f9_norm(f9_sub(hi, lo));
    e[0] = lo;
    e[1] = f9_norm_reduce(f9_add(hi, dn));
    e[2] = f9_norm_reduce(f9_add(e[1], dn));
}

struct IntRow {
    int64_t z, zp, ns;
};
__device__ __forceinline__ IntRow int_row(int64_t z, int nbits, int r_bits) {
    IntRow r;
    r.z = z;
    r.zp = rescale_half_up(z, r_bits);
    r.ns = 1 - ((z >> (nbits - 1)) & 1);
    return r;
}

// The four input claims from the integers (same bounds as round 0 below): dot products of the
// equality tables as built with Z, (1 - sign) Z', G_A, (1 - sign) G_A'; also the range check.
// sum_i H[ih] L[il] c_i = sum_ih H[ih] (sum_il L[il] c_i): a block takes a contiguous range of i and a
// thread keeps the inner sums (9 x 2 limb products, no reduction) for as long as its ih stays the
// same; when it changes the sums are reduced and multiplied by H[ih].
__global__ __launch_bounds__(ZK_BLOCK) void k_zk_prepare_int(PrepArgs a) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    uint64_t cols[4][11];
    F9 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        acc[q] = f9_zero();
#pragma unroll
        for (int c = 0; c < 11; ++c) cols[q][c] = 0;
    }
    bool bad = false;
    const int lb = a.sp.lb;
    const uint64_t per = ((a.D + gridDim.x - 1) / gridDim.x + ZK_BLOCK - 1) / ZK_BLOCK * ZK_BLOCK;
    const uint64_t i0 = blockIdx.x * per, i1 = i0 + per < a.D ? i0 + per : a.D;
    const uint64_t none = ~(uint64_t)0;
    uint64_t cur = none;
    auto flush = [&](uint64_t ih) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (q >= 2 && !a.ga) continue;
            acc[q] = f9_norm_reduce(f9_add(acc[q], f9_mul(f9tab_ld(a.sp.H[q], ih), cols11_value(cols[q]))));
#pragma unroll
            for (int c = 0; c < 11; ++c) cols[q][c] = 0;
        }
    };
    for (uint64_t i = i0 + threadIdx.x; i < i1; i += ZK_BLOCK) {
        const uint64_t ih = i >> lb, il = i & (((uint64_t)1 << lb) - 1);
        if (ih != cur) {
            if (cur != none) flush(cur);
            cur = ih;
        }
        const int64_t z = a.z[i];
        bad |= !in_range(z, a.nbits);
        const IntRow rz = int_row(z, a.nbits, a.r_bits);
        cols11_mac_signed(cols[0], f9tab_ld(a.sp.L[0], il), rz.z);
        cols11_mac_signed(cols[1], f9tab_ld(a.sp.L[1], il), rz.ns * rz.zp);
        cols11_carry(cols[0]);
        cols11_carry(cols[1]);
        if (a.ga) {
            const int64_t g = a.ga[i];
            bad |= !in_range(g, a.nbits);
            cols11_mac_signed(cols[2], f9tab_ld(a.sp.L[2], il), g);
            cols11_mac_signed(cols[3], f9tab_ld(a.sp.L[3], il), rz.ns * rescale_half_up(g, a.r_bits));
            cols11_carry(cols[2]);
            cols11_carry(cols[3]);
        }
    }
    if (cur != none) flush(cur);
    if (bad) atomicOr(&a.st->err, 1u);
    const Fr s = block_sum_lazy<4>(acc, red);
    if (threadIdx.x < 4) a.part[(uint64_t)blockIdx.x * 4 + threadIdx.x] = s;
}

// Round 0.  Bounds: |Z| < 2^55, so a line value |3 hi - 2 lo| < 2^57.4; |Z'| <= 2^54, the line of
// 1 - sign is within [-2, 3]: their product is below 2^58.
// The pair (b, b + m) differs in the leading variable, which lies in H: with b = (bh, bl),
//   sum_b beta(x, b) c_b(x) = sum_bh Hline_bh(x) (sum_bl L[bl] c_b(x)),
// so a block takes one equation and a contiguous range of b, a thread keeps the inner sums for
// as long as its bh stays the same, and only then reduces them and multiplies by the line of H.
__device__ __forceinline__ void lin0_int_body(const LinArgs& a, const unsigned bx) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    const unsigned nbq = a.eq_blocks, e = bx / nbq, q = bx % nbq;
    const uint64_t m = a.m;
    const int lb = a.sp.lb;
    const uint64_t hh = m >> lb;                  // H entries per half
    const uint64_t per = ((m + nbq - 1) / nbq + ZK_BLOCK - 1) / ZK_BLOCK * ZK_BLOCK;
    const uint64_t b0 = q * per, b1 = b0 + per < m ? b0 + per : m;
    const F9Tab H = a.sp.H[e], L = a.sp.L[e];
    uint64_t cols[3][11];
    F9 tot[3];
#pragma unroll
    for (int x = 0; x < 3; ++x) {
        tot[x] = f9_zero();
#pragma unroll
        for (int c = 0; c < 11; ++c) cols[x][c] = 0;
    }
    const uint64_t none = ~(uint64_t)0;
    uint64_t cur = none;
    auto flush = [&](uint64_t bh) {
        F9 hl[3];
        line3_reduced(f9tab_ld(H, bh), f9tab_ld(H, bh + hh), hl);
#pragma unroll
        for (int x = 0; x < 3; ++x) {
            tot[x] = f9_norm_reduce(f9_add(tot[x], f9_mul(hl[x], cols11_value(cols[x]))));
#pragma unroll
            for (int c = 0; c < 11; ++c) cols[x][c] = 0;
        }
    };
    for (uint64_t b = b0 + threadIdx.x; b < b1; b += ZK_BLOCK) {
        const uint64_t bh = b >> lb;
        if (bh != cur) {
            if (cur != none) flush(cur);
            cur = bh;
        }
        const IntRow zl = int_row(a.z[b], a.nbits, a.r_bits), zh = int_row(a.z[b + m], a.nbits, a.r_bits);
        int64_t vl, vh;   // the value whose line is taken, before the factor 1 - sign
        if (e == 0) {
            vl = zl.z;
            vh = zh.z;
        } else if (e == 1) {
            vl = zl.zp;
            vh = zh.zp;
        } else {
            const int64_t gl = a.ga[b], gh = a.ga[b + m];
            vl = e == 2 ? gl : rescale_half_up(gl, a.r_bits);
            vh = e == 2 ? gh : rescale_half_up(gh, a.r_bits);
        }
        const F9 lv = f9tab_ld(L, b & (((uint64_t)1 << lb) - 1));
#pragma unroll
        for (int x = 0; x < 3; ++x) {
            const int64_t xx = x ? x + 1 : 0;
            int64_t c = vl + xx * (vh - vl);
            if (e & 1) c *= zl.ns + xx * (zh.ns - zl.ns);
            cols11_mac_signed(cols[x], lv, c);
            cols11_carry(cols[x]);
        }
    }
    if (cur != none) flush(cur);
    const Fr s = block_sum_lazy<3>(tot, red);
    Fr* pp = a.part + (uint64_t)bx * 4;
    if (threadIdx.x < 3) pp[threadIdx.x ? threadIdx.x + 1 : 0] = s;
    else if (threadIdx.x == 3) pp[1] = fr_zero();
}

// Round 1: v0 is bound on the way; the equality tables come from their two factors (H already
// folded), the value tables from the integers and are written out folded (length 2m).  As in
// round 0 a block takes one equation and a contiguous range of pair indices, and the sums are
// grouped by the H index: with b = (bh, bl) and u = L[bl] value,
//   "in" equations:  sum_b beta(x, b) q_b(x)        = sum_bh Hline_bh(x) line(sum u_lo, sum u_hi)(x),
//   "out" equations: sum_b beta(x, b) ns_b(x) q_b(x) = sum_bh Hline_bh(x) sum ns_b(x) line(u_lo, u_hi)(x),
// so a pair costs two products (five with the factor 1 - sign) next to the two folds of its value
// table, and the line of H is multiplied in once per run.  Equation 1 also writes the folded
// 1 - sign table; the folded equality tables are written only if the next round reads them from
// memory (write_eq).
__device__ __forceinline__ void lin1_int_body(const LinArgs& a, const unsigned bx) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    __shared__ F9 kf[4];     // R^2, -R^2, v0 R^2, -v0 R^2
    __shared__ F9 kns[4];    // 1 - sign folded, by (bit at x0 = 0) + 2 (bit at x0 = 1): 0, 1 - v0, v0, 1
    if (threadIdx.x < 4) {
        const Fr v0 = *a.chal, r2 = fr_const(frc::R2), one = fr_one();
        const Fr c = threadIdx.x < 2 ? r2 : fr_mul(v0, r2);
        kf[threadIdx.x] = fr_unpack((threadIdx.x & 1) ? fr_neg(c) : c);
        kns[threadIdx.x] = fr_unpack(threadIdx.x == 0 ? fr_zero() : threadIdx.x == 1 ? fr_sub(one, v0)
                                     : threadIdx.x == 2 ? v0 : one);
    }
    __syncthreads();
    const unsigned nbq = a.eq_blocks, e = bx / nbq, q = bx % nbq;
    const bool with_ns = e & 1;
    const uint64_t m = a.m;
    const int lb = a.sp.lb;
    const uint64_t hh = m >> lb;                  // H entries per half; 0 (D < 16): the pair differs inside L
    const uint64_t per = ((m + nbq - 1) / nbq + ZK_BLOCK - 1) / ZK_BLOCK * ZK_BLOCK;
    const uint64_t b0 = q * per, b1 = b0 + per < m ? b0 + per : m;
    const F9Tab H = a.sp.H[e], L = a.sp.L[e];
    const F9Tab vt = a.tabs.t[e == 0 ? T_Z : e == 1 ? T_ZP : e == 2 ? T_GA : T_GAP];
    const F9Tab et = a.tabs.t[e == 0 ? T_BZ : e == 1 ? T_BA : e == 2 ? T_BGA : T_BGZ];
    F9 acc[3], tot[3];   // acc: "in": sums of u_lo, u_hi (third unused); "out": sums at x = 0, 2, 3
#pragma unroll
    for (int x = 0; x < 3; ++x) acc[x] = tot[x] = f9_zero();
    const uint64_t none = ~(uint64_t)0;
    uint64_t cur = none;
    auto flush = [&](uint64_t bh) {
        F9 hl[3], s[3];
        line3<true>(f9tab_ld(H, bh), f9tab_ld(H, bh + hh), hl);
        if (with_ns) {
#pragma unroll
            for (int x = 0; x < 3; ++x) s[x] = acc[x];
        } else {
            line3<true>(acc[0], acc[1], s);
        }
#pragma unroll
        for (int x = 0; x < 3; ++x) {
            tot[x] = f9_norm_reduce(f9_add(tot[x], f9_mul(hl[x], s[x])));
            acc[x] = f9_zero();
        }
    };
    for (uint64_t b = b0 + threadIdx.x; b < b1; b += ZK_BLOCK) {
        const uint64_t bh = b >> lb;
        if (hh != 0 && bh != cur) {
            if (cur != none) flush(cur);
            cur = bh;
        }
        IntRow r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = int_row(a.z[b + i * m], a.nbits, a.r_bits);
        int64_t v4[4];   // the value rows: b, b + 2m fold into lo; b + m, b + 3m into hi
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (e < 2) {
                v4[i] = e == 0 ? r[i].z : r[i].zp;
            } else {
                const int64_t g = a.ga[b + i * m];
                v4[i] = e == 2 ? g : rescale_half_up(g, a.r_bits);
            }
        }
        const F9 lo = fold_ints(kf, v4[0], v4[2]), hi = fold_ints(kf, v4[1], v4[3]);
        f9tab_st(vt, b, lo);
        f9tab_st(vt, b + m, hi);
        const uint64_t mask = ((uint64_t)1 << lb) - 1;
        const F9 llo = f9tab_ld(L, b & mask), lhi = hh ? llo : f9tab_ld(L, (b + m) & mask);
        if (hh == 0) {
            // D < 16: the pair differs inside L, so the equality line is not a multiple of one L
            // entry; each pair is worked out by itself (cur stays unset: nothing to flush)
            const F9 h0 = f9tab_ld(H, 0);
            const F9 plo = f9_mul(h0, llo), phi = f9_mul(h0, lhi);
            if (a.write_eq) {
                f9tab_st(et, b, plo);
                f9tab_st(et, b + m, phi);
            }
            F9 p[3], qv[3];
            line3<true>(plo, phi, p);
            line3<false>(lo, hi, qv);
            if (with_ns) {
                const F9 nlo = kns[(int)(r[0].ns + 2 * r[2].ns)], nhi = kns[(int)(r[1].ns + 2 * r[3].ns)];
                if (e == 1) {
                    f9tab_st(a.tabs.t[T_NS], b, nlo);
                    f9tab_st(a.tabs.t[T_NS], b + m, nhi);
                }
                F9 ns[3];
                line3<false>(nlo, nhi, ns);
#pragma unroll
                for (int x = 0; x < 3; ++x) tot[x] = f9_norm_reduce(f9_add(tot[x], f9_mul(f9_mul(p[x], ns[x]), qv[x])));
            } else {
#pragma unroll
                for (int x = 0; x < 3; ++x) tot[x] = f9_norm_reduce(f9_add(tot[x], f9_mul(p[x], qv[x])));
            }
            continue;
        }
        const F9 ulo = f9_mul(llo, lo), uhi = f9_mul(lhi, hi);     // normal, below 2 r
        if (a.write_eq) {
            f9tab_st(et, b, f9_mul(f9tab_ld(H, bh), llo));
            f9tab_st(et, b + m, f9_mul(f9tab_ld(H, bh + hh), lhi));
        }
        if (with_ns) {
            const F9 nlo = kns[(int)(r[0].ns + 2 * r[2].ns)], nhi = kns[(int)(r[1].ns + 2 * r[3].ns)];
            if (e == 1) {
                f9tab_st(a.tabs.t[T_NS], b, nlo);
                f9tab_st(a.tabs.t[T_NS], b + m, nhi);
            }
            F9 ns[3], uq[3];
            line3<false>(nlo, nhi, ns);
            line3<true>(ulo, uhi, uq);
#pragma unroll
            for (int x = 0; x < 3; ++x) acc[x] = f9_norm_reduce(f9_add(acc[x], f9_mul(uq[x], ns[x])));
        } else {
            acc[0] = f9_norm_reduce(f9_add(acc[0], ulo));
            acc[1] = f9_norm_reduce(f9_add(acc[1], uhi));
        }
    }
    if (cur != none) flush(cur);
    {
        const Fr s = block_sum_lazy<3>(tot, red);
        Fr* pp = a.part + (uint64_t)bx * 4;
        if (threadIdx.x < 3) pp[threadIdx.x ? threadIdx.x + 1 : 0] = s;
        else if (threadIdx.x == 3) pp[1] = fr_zero();
    }
}

// The same sum for a round with few pairs, where one thread per pair would leave a chain
// of 36 products: a block takes 16 pairs; first a thread per (table, pair) folds and leaves
// the pair in LDS, then a thread per (evaluation point, equation, pair) multiplies, with
// wave w summing the point x = 0, 2, 3 [w] by itself.
constexpr int LIN_SMALL_PAIRS = 16;

// value at x = 0, 2, 3 (xi = 0, 1, 2) of the line through (lo, hi); limbs below 2^30.6
__device__ __forceinline__ F9 line_at(const F9& lo, const F9& hi, int xi) {
    if (xi == 0) return lo;
    const F9 dn = f9_norm(f9_sub(hi, lo));
    F9 e = f9_add(hi, dn);
    if (xi == 2) e = f9_add(e, dn);
    return e;
}

template <bool FOLD>
__device__ __forceinline__ void lin_body_small(const LinArgs& a, const unsigned bx) {
    // tables in the order NS | BZ Z | BA ZP | BGA GA | BGZ GAP
    __shared__ uint32_t pairs[9][2][9][LIN_SMALL_PAIRS];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int ntab = a.has_ga ? 9 : 5, nterm = a.has_ga ? 4 : 2;
    const uint64_t m = a.m;
    F9 v = f9_zero();
    if (FOLD) v = fr_unpack(*a.chal);
    {
        const int ti = tid / LIN_SMALL_PAIRS, bl = tid % LIN_SMALL_PAIRS;
        const uint64_t b = (uint64_t)bx * LIN_SMALL_PAIRS + bl;
        if (ti < ntab) {
            F9 lo = f9_zero(), hi = f9_zero();
            if (b < m) {
                const int which = ti == 0 ? T_NS : ti == 1 ? T_BZ : ti == 2 ? T_Z : ti == 3 ? T_BA : ti == 4 ? T_ZP
                                : ti == 5 ? T_BGA : ti == 6 ? T_GA : ti == 7 ? T_BGZ : T_GAP;
                lin_pair<FOLD>(a.tabs.t[which], b, m, v, lo, hi);
            }
#pragma unroll
            for (int l = 0; l < 9; ++l) {
                pairs[ti][0][l][bl] = lo.v[l];
                pairs[ti][1][l][bl] = hi.v[l];
            }
        }
    }
    __syncthreads();
    F9 prod = f9_zero();
    {
        const int term = lane / LIN_SMALL_PAIRS, bl = lane % LIN_SMALL_PAIRS;
        const uint64_t b = (uint64_t)bx * LIN_SMALL_PAIRS + bl;
        if (wave < 3 && term < nterm && b < m) {
            const int tp = 1 + 2 * term, tq = 2 + 2 * term;   // beta table, value table
            F9 lo, hi;
#pragma unroll
            for (int l = 0; l < 9; ++l) {
                lo.v[l] = pairs[tp][0][l][bl];
                hi.v[l] = pairs[tp][1][l][bl];
            }
            prod = f9_norm(line_at(lo, hi, wave));
            if (term & 1) {   // the equations with (1 - sign)
#pragma unroll
                for (int l = 0; l < 9; ++l) {
                    lo.v[l] = pairs[0][0][l][bl];
                    hi.v[l] = pairs[0][1][l][bl];
                }
                prod = f9_mul(prod, line_at(lo, hi, wave));
            }
#pragma unroll
            for (int l = 0; l < 9; ++l) {
                lo.v[l] = pairs[tq][0][l][bl];
                hi.v[l] = pairs[tq][1][l][bl];
            }
            prod = f9_norm_reduce(f9_mul(prod, line_at(lo, hi, wave)));
        }
    }
    const F9 s = wave_sum_lazy(prod);
    Fr* pp = a.part + (uint64_t)bx * 4;
    if (wave < 3 && lane == 0) pp[wave ? wave + 1 : 0] = f9_to_fr(s);
    else if (tid == 255) pp[1] = fr_zero();
}

// ---------------------------------------------------------------------------
// i-rounds, binarity terms
// ---------------------------------------------------------------------------
struct BinArgs {
    const int64_t* z;      // round 0 / materialise only
    const int64_t* ga;
    uint32_t* aux;         // lazy-limb planes: entry (k, j, i), limb l at ((k*nbits + j)*9 + l)*ps + i
    uint64_t ps;
    int nbits;
    int has_ga;
    uint64_t m;            // pairs this round
    int jc;                // columns per thread
    const Fr* chal;
    F9Tab bI;              // beta_I, lazy limbs: round 0 the table as built; later the entries for
                           // both values of the previous variable (length 4m)
    F9Tab bI_out;          // rounds >= 1: receives the pair folded with vprev (length 2m)
    const Fr* vprev;       // rounds >= 1: challenge of the previous round
    int ksplit;            // column chunk = by / 2 and slice = by % 2 (few rows: more threads)
    const Fr* bJ;          // J entries
    const Fr* rp;          // r'
    int split;             // rounds 0, 1: beta_I(i) = sH[i >> s_lb] sL[i & (2^s_lb - 1)] (sH bound as far as needed)
    F9Tab sH, sL;
    int s_lb;
    // per pair index the sums over the columns SA = sum beta_J p(lo), SC = sum beta_J p(hi),
    // SD = sum beta_J (hi - lo)^2, p(a) = a^2 - a, handed from one round to the next
    // (entry (chunk, b) at index chunk * pairs + b; the chunks of a pair index add up)
    F9Tab ps_in[3];        // what the previous round left (binp_body)
    int ps_in_chunks;
    F9Tab ps_out[3];       // written if ps_write
    int ps_write;
    Fr* part;              // partials of this kernel
};

__device__ __forceinline__ FrTab aux_col(const BinArgs& a, int k, int j) {
    FrTab t;
    t.p = a.aux + (uint64_t)(k * a.nbits + j) * 8 * a.ps;
    t.ps = a.ps;
    return t;
}

// sum of beta_J (lazy limbs, LDS) over the set bits of mask; normal on return
__device__ __forceinline__ F9 masked_sum9(const F9* sbj, uint64_t mask) {
    F9 s = f9_zero();
    int pending = 0;
    while (mask) {
        const int j = __builtin_ctzll(mask);
        mask &= mask - 1;
        s = f9_add(s, sbj[j]);
        if (++pending == 4) {
            pending = 0;
            s = f9_norm(s);
        }
    }
    return f9_norm(s);
}

// Sums of beta_J over column sets by table: the columns are cut into groups of BJ_BITS and
// tab[g][e] holds the sum of beta_J(BJ_BITS g + i) over the set bits i of e (normal, below
// BJ_BITS r), so a masked sum is one table entry per group and the same work for every lane.
constexpr int BJ_BITS = 7;
constexpr int BJ_MAXG = (64 + BJ_BITS - 1) / BJ_BITS;
constexpr int BJ_TAB_WORDS = BJ_MAXG * (1 << BJ_BITS) * 9;

// sbj: beta_J as lazy limbs (64 entries, zero beyond nbits); all threads of the block
__device__ __forceinline__ void bj_tables_build(uint32_t* tab, const F9* sbj, int groups) {
    for (int idx = threadIdx.x; idx < groups << BJ_BITS; idx += blockDim.x) {
        const int g = idx >> BJ_BITS, e = idx & ((1 << BJ_BITS) - 1);
        F9 s = f9_zero();
#pragma unroll
        for (int i = 0; i < BJ_BITS; ++i)
            if (((e >> i) & 1) && BJ_BITS * g + i < 64) s = f9_add(s, sbj[BJ_BITS * g + i]);
        s = f9_norm(s);
#pragma unroll
        for (int l = 0; l < 9; ++l) tab[idx * 9 + l] = s.v[l];
    }
}

// sum of beta_J over the set bits of mask: normal, below 64 r
__device__ __forceinline__ F9 bj_masked_sum(const uint32_t* tab, uint64_t mask, int groups) {
    F9 s = f9_zero();
#pragma unroll
    for (int g = 0; g < BJ_MAXG; ++g) {
        if (g < groups) {
            const uint32_t* e = tab + ((g << BJ_BITS) + (uint32_t)((mask >> (BJ_BITS * g)) & ((1u << BJ_BITS) - 1))) * 9;
#pragma unroll
            for (int l = 0; l < 9; ++l) s.v[l] += e[l];
        }
        if (g == 6) s = f9_norm(s);   // seven entries with limbs below 2^29 each so far
    }
    s = f9_norm(s);
    // keep the scheduler from starting the next sum's loads before this one is consumed: with
    // several sums in flight the registers run out
    __builtin_amdgcn_sched_barrier(0);
    return s;
}

// Round 0: both halves are bits, a(x)^2 - a(x) = (x^2 - x) [lo != hi]; contributes
// 2 beta_I(2, i') C(i') at x = 2 and 6 beta_I(3, i') C(i') at x = 3,
// C = sum_j beta_J(j) ([z bits differ] + r' [g bits differ]).
__device__ __forceinline__ void bin0_body(const BinArgs& a, const unsigned bx, const unsigned gx) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    __shared__ F9 sbj[2][64];   // beta_J, and r' beta_J for the second slice
    const int tid = threadIdx.x;
    if (tid < 128) {
        const int j = tid & 63, k = tid >> 6;
        F9 x = f9_zero();
        if (j < a.nbits) x = fr_unpack(k == 0 ? a.bJ[j] : fr_mul(*a.rp, a.bJ[j]));
        sbj[k][j] = x;
    }
    __syncthreads();
    F9 acc[2];
    acc[0] = f9_zero();
    acc[1] = f9_zero();
    const uint64_t m = a.m;
    const uint64_t keep = a.nbits >= 64 ? ~(uint64_t)0 : (((uint64_t)1 << a.nbits) - 1);
    if (a.split) {
        // beta_I(x, b) = Hline_bh(x) L[bl]: a block takes a contiguous range of b and a thread adds up
        // L[bl] C(b) for as long as its bh stays the same, then multiplies by the line of H
        __shared__ uint32_t bjt[BJ_TAB_WORDS];   // masked sums of beta_J by table; slice 1 takes r' afterwards
        const int groups = (a.nbits + BJ_BITS - 1) / BJ_BITS;
        bj_tables_build(bjt, sbj[0], groups);
        __syncthreads();
        const F9 rp9 = fr_unpack(*a.rp);
        const int lb = a.s_lb;
        const uint64_t hh = m >> lb;
        const uint64_t per = ((m + gx - 1) / gx + ZK_BLOCK - 1) / ZK_BLOCK * ZK_BLOCK;
        const uint64_t b0 = bx * per, b1 = b0 + per < m ? b0 + per : m;
        const uint64_t none = ~(uint64_t)0;
        uint64_t cur = none;
        F9 u = f9_zero();
        auto flush = [&](uint64_t bh) {
            const F9 lo = f9tab_ld(a.sH, bh), hi = f9tab_ld(a.sH, bh + hh);
            const F9 dn = f9_norm(f9_sub(hi, lo));
            const F9 b2 = f9_norm(f9_add(hi, dn)), b3 = f9_norm(f9_add(b2, dn));
            acc[0] = f9_norm_reduce(f9_add(acc[0], f9_mul(b2, u)));
            acc[1] = f9_norm_reduce(f9_add(acc[1], f9_mul(b3, u)));
            u = f9_zero();
        };
        for (uint64_t b = b0 + tid; b < b1; b += ZK_BLOCK) {
            const uint64_t bh = b >> lb;
            if (bh != cur) {
                if (cur != none) flush(cur);
                cur = bh;
            }
            const uint64_t dz = ((uint64_t)a.z[b] ^ (uint64_t)a.z[b + m]) & keep;
            F9 c = bj_masked_sum(bjt, dz, groups);               // normal, below 64 r
            if (a.has_ga) {
                const uint64_t dg = ((uint64_t)a.ga[b] ^ (uint64_t)a.ga[b + m]) & keep;
                c = f9_add(c, f9_mul(rp9, bj_masked_sum(bjt, dg, groups)));   // limbs below 2^30
            }
            u = f9_norm_reduce(f9_add(u, f9_mul(f9tab_ld(a.sL, b & (((uint64_t)1 << lb) - 1)), c)));
        }
        if (cur != none) flush(cur);
    } else {
        for (uint64_t b = bx * (uint64_t)blockDim.x + tid; b < m; b += (uint64_t)gx * blockDim.x) {
            const uint64_t dz = ((uint64_t)a.z[b] ^ (uint64_t)a.z[b + m]) & keep;
            F9 c = masked_sum9(sbj[0], dz);                      // normal, below 64 r
            if (a.has_ga) {
                const uint64_t dg = ((uint64_t)a.ga[b] ^ (uint64_t)a.ga[b + m]) & keep;
                c = f9_add(c, masked_sum9(sbj[1], dg));          // limbs below 2^30
            }
            // round 0: the table is as built, fully reduced; line at x = 2, 3, normal
            const F9 lo = f9tab_ld(a.bI, b), hi = f9tab_ld(a.bI, b + m);
            const F9 dn = f9_norm(f9_sub(hi, lo));
            const F9 b2 = f9_norm(f9_add(hi, dn)), b3 = f9_norm(f9_add(b2, dn));
            acc[0] = f9_norm_reduce(f9_add(acc[0], f9_mul(b2, c)));
            acc[1] = f9_norm_reduce(f9_add(acc[1], f9_mul(b3, c)));
        }
    }
    // (x^2 - x) = 2 at x = 2 and 6 at x = 3
    acc[0] = f9_norm_reduce(f9_add(acc[0], acc[0]));
    const F9 a3 = f9_add(acc[1], acc[1]);
    acc[1] = f9_norm_reduce(f9_add(f9_add(a3, a3), a3));     // limbs below 6 * 2^29
    const Fr s = block_sum_lazy<2>(acc, red);
    Fr* p = a.part + (uint64_t)bx * 4;
    if (tid < 2) p[2 + tid] = s;
    else if (tid < 4) p[tid - 2] = fr_zero();
}

// ---- rounds >= 1 work on field elements; the first challenges are bound by table look-up ----
//
// aux is binary, so after binding x0 = v0 an entry is one of four values, selected by the
// two bits it interpolates: A(b_lo, b_hi) = b_lo + v0 (b_hi - b_lo), code = b_lo + 2 b_hi:
//   code 0 -> 0, 1 -> 1 - v0, 2 -> v0, 3 -> 1.
// Round 1 (variable x1) pairs two such entries; its summand is a quadratic form in the four bits
// that an entry pair interpolates, with coefficients that are constants of the round, so the
// round needs no table in memory at all: sums of beta_J over column sets chosen by the bits, and
// five products per (i, slice) (bin1_body).  After v1 the entry is one of 16 values (k_zk_mat2
// writes them out, D/4 rows); later rounds fold as usual.

__device__ __forceinline__ F9Tab aux_col9(const BinArgs& a, int k, int j) {
    F9Tab t;
    t.p = a.aux + (uint64_t)(k * a.nbits + j) * 9 * a.ps;
    t.ps = a.ps;
    return t;
}

__device__ __forceinline__ Fr bit_pair_value(int code, const Fr& v, const Fr& one) {
    return code == 0 ? fr_zero() : code == 3 ? one : code == 2 ? v : fr_sub(one, v);
}

// beta_I in rounds t >= 1: the source still has the entries for both values of the previous
// variable (length 4m); bind the previous challenge, leave the folded pair in the other buffer
// for the next round (every column chunk writes the same values), return the line at 0, 2, 3
__device__ __forceinline__ void beta_line_fold(const BinArgs& a, uint64_t b, uint64_t m, const F9& vprev, F9 e[3]) {
    F9 lo, hi;
    if (a.split) {   // the H factor is folded already
        lo = split_entry(a.sH, a.sL, a.s_lb, b);
        hi = split_entry(a.sH, a.sL, a.s_lb, b + m);
    } else {
        const F9 t0 = f9tab_ld(a.bI, b), t1 = f9tab_ld(a.bI, b + m);
        const F9 t2 = f9tab_ld(a.bI, b + 2 * m), t3 = f9tab_ld(a.bI, b + 3 * m);
        lo = f9_norm_reduce(f9_add(t0, f9_mul(f9_sub(t2, t0), vprev)));
        hi = f9_norm_reduce(f9_add(t1, f9_mul(f9_sub(t3, t1), vprev)));
    }
    f9tab_st(a.bI_out, b, lo);
    f9tab_st(a.bI_out, b + m, hi);
    const F9 dn = f9_norm(f9_sub(hi, lo));
    e[0] = lo;
    e[1] = f9_norm(f9_add(hi, dn));
    e[2] = f9_norm(f9_add(e[1], dn));
}

// Column sums from round to round.  With p(a) = a^2 - a the summand of a pair (lo, hi) is
//   q(X) = (1 - X) p(lo) + X p(hi) - X (1 - X) (hi - lo)^2,
// so the sums over the columns SA = sum beta_J p(lo), SC = sum beta_J p(hi), SD = sum beta_J (hi - lo)^2
// give the round's G(0) = SA, G(2) = -SA + 2 SC + 2 SD, G(3) = -2 SA + 3 SC + 6 SD, and at X = v (the
// challenge bound next) what p of the folded entries sums to.  A pair of the next round folds the
// pairs b and b + m of this one, hence its SA' = (1 - v) SA_b + v SC_b - v (1 - v) SD_b and SC' the
// same at b + m: only SD' needs the columns again.
struct PsumConsts {
    F9 u1, v, nvv;   // 1 - v, v, v^2 - v
};
__device__ __forceinline__ PsumConsts psum_consts(const Fr* vp) {
    const Fr vf = *vp;
    PsumConsts k;
    k.u1 = fr_unpack(fr_sub(fr_one(), vf));
    k.v = fr_unpack(vf);
    k.nvv = fr_unpack(fr_sub(fr_sqr(vf), vf));
    return k;
}
// SA', SC' of pair index b (of m) from what the previous round left (2m pairs, ps_in_chunks chunks
// that add up); both normal and below 2.41 r
__device__ __forceinline__ void psum_bind(const BinArgs& a, uint64_t b, uint64_t m, const PsumConsts& k, F9& sa, F9& sc) {
    F9 in[2][3];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int q = 0; q < 3; ++q) in[h][q] = f9_zero();
    for (int c = 0; c < a.ps_in_chunks; ++c) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int q = 0; q < 3; ++q)
                in[h][q] = f9_norm_reduce(f9_add(in[h][q], f9tab_ld(a.ps_in[q], (uint64_t)c * 2 * m + b + h * m)));
    }
    // three products below 2.41 r^2 each
    sa = f9_norm_reduce(f9_add(f9_add(f9_mul(k.u1, in[0][0]), f9_mul(k.v, in[0][1])), f9_mul(k.nvv, in[0][2])));
    sc = f9_norm_reduce(f9_add(f9_add(f9_mul(k.u1, in[1][0]), f9_mul(k.v, in[1][1])), f9_mul(k.nvv, in[1][2])));
}
// the round's G(0), G(2), G(3) times the beta_I line, added to tot; sa below 2.6 r, all normal with
// limbs below 2^29 (at most eight are added between carry passes)
__device__ __forceinline__ void psum_accumulate(F9 tot[3], const F9 bi[3], const F9& sa, const F9& sc, const F9& sd) {
    const F9 sc2 = f9_add(sc, sc), sd2 = f9_add(sd, sd);
    const F9 g2 = f9_norm(f9_sub(f9_add(sc2, sd2), sa));                             // -SA + 2 SC + 2 SD
    const F9 h3 = f9_norm(f9_add(f9_add(sc2, sc), f9_add(sd2, sd2)));                // 3 SC + 4 SD
    const F9 g3 = f9_norm(f9_sub(f9_sub(f9_add(h3, sd2), sa), sa));                  // ... + 2 SD - 2 SA
    tot[0] = f9_norm_reduce(f9_add(tot[0], f9_mul(bi[0], sa)));
    tot[1] = f9_norm_reduce(f9_add(tot[1], f9_mul(bi[1], g2)));
    tot[2] = f9_norm_reduce(f9_add(tot[2], f9_mul(bi[2], g3)));
}
__device__ __forceinline__ void psum_store(const BinArgs& a, uint64_t at, const F9& sa, const F9& sc, const F9& sd) {
    f9tab_st(a.ps_out[0], at, sa);
    f9tab_st(a.ps_out[1], at, sc);
    f9tab_st(a.ps_out[2], at, sd);
}

// Round 1 on the integers.  m = D/4 quadruples of rows (i'', i''+m | i''+2m, i''+3m) = (x0, x1) in
// {(0,0), (0,1), (1,0), (1,1)}; bit j of row (x0, x1) is B_{x0,x1}(j).  With x0 bound to v0 the
// entry that the round interpolates is
//   e_j(X) = sum_{x0,x1} chi_{x0} w_{x1}(X) B_{x0,x1}(j),  chi = (1 - v0, v0),  w(X) = (1 - X, X),
// a combination of bits whose coefficients add up to one, hence
//   e^2 - e = - sum over unordered pairs of rows of (coefficient product) [the two bits differ].
// Summed over the columns with beta_J that is
//   sum_j beta_J(j) q_j(X) = -[(1-X)^2 A + X^2 C + X(1-X) B],
//   A = chi0 chi1 S(B00 ^ B10),  C = chi0 chi1 S(B01 ^ B11),
//   B = chi0^2 S(B00 ^ B01) + chi0 chi1 (S(B00 ^ B11) + S(B10 ^ B01)) + chi1^2 S(B10 ^ B11),
// S(mask) = sum of beta_J over the set bits: six masked sums and five products per
// (quadruple, slice), whatever the bits are.  A and C are accumulated with the negated constant
// (A' = -A, C' = -C): G(0) = A', G(2) = A' + 4 C' + 2 B, G(3) = 4 A' + 9 C' + 6 B.  Writes partial sums for x = 0, 2, 3
// (x = 1 comes from the claim).
__device__ __forceinline__ void bin1_body(const BinArgs& a, const unsigned bx, const unsigned gx) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    __shared__ F9 sbj[64];
    __shared__ uint32_t bjt[BJ_TAB_WORDS];
    __shared__ F9 kc[2][4];   // [slice][-chi0 chi1, chi0^2, chi0 chi1, chi1^2]; slice 1 carries r'
    const int tid = threadIdx.x;
    const int groups = (a.nbits + BJ_BITS - 1) / BJ_BITS;
    if (tid < 64) sbj[tid] = tid < a.nbits ? fr_unpack(a.bJ[tid]) : f9_zero();
    if (tid >= 64 && tid < 72) {
        const int k = (tid - 64) >> 2, q = (tid - 64) & 3;
        const Fr v0 = *a.chal, u0 = fr_sub(fr_one(), v0);
        Fr c = q == 1 ? fr_sqr(u0) : q == 3 ? fr_sqr(v0) : fr_mul(u0, v0);
        if (q == 0) c = fr_neg(c);
        if (k == 1) c = fr_mul(*a.rp, c);
        kc[k][q] = fr_unpack(c);
    }
    __syncthreads();
    bj_tables_build(bjt, sbj, groups);
    __syncthreads();
    const uint64_t m = a.m;
    const F9 vprev9 = fr_unpack(*a.vprev);
    const uint64_t keep = a.nbits >= 64 ? ~(uint64_t)0 : (((uint64_t)1 << a.nbits) - 1);
    F9 tot[3];
#pragma unroll
    for (int x = 0; x < 3; ++x) tot[x] = f9_zero();
    for (uint64_t b = bx * (uint64_t)blockDim.x + tid; b < m; b += (uint64_t)gx * blockDim.x) {
        // rows of the quadruple, both slices
        uint64_t w[2][4];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int64_t* src = k == 0 ? a.z : a.ga;
#pragma unroll
            for (int q = 0; q < 4; ++q) w[k][q] = (k == 0 || a.has_ga) ? (uint64_t)src[b + q * m] & keep : 0;
        }
        // w[k][0] = B00, [1] = B01, [2] = B10, [3] = B11 (x0 selects the half, x1 the quarter).
        // Every masked sum is normal and below 64 r; one accumulator at a time.
        F9 red3[3];   // A', C', B
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            uint64_t cols[17];
#pragma unroll
            for (int c = 0; c < 17; ++c) cols[c] = 0;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                if (k == 1 && !a.has_ga) break;
                if (t == 0) {
                    f9_cols_mac(cols, kc[k][0], bj_masked_sum(bjt, w[k][0] ^ w[k][2], groups));
                } else if (t == 1) {
                    f9_cols_mac(cols, kc[k][0], bj_masked_sum(bjt, w[k][1] ^ w[k][3], groups));
                } else {
                    f9_cols_mac(cols, kc[k][1], bj_masked_sum(bjt, w[k][0] ^ w[k][1], groups));
                    const F9 cross = f9_norm(f9_add(bj_masked_sum(bjt, w[k][0] ^ w[k][3], groups),
                                                    bj_masked_sum(bjt, w[k][2] ^ w[k][1], groups)));
                    f9_cols_mac(cols, kc[k][2], cross);
                    f9_cols_mac(cols, kc[k][3], bj_masked_sum(bjt, w[k][2] ^ w[k][3], groups));
                    f9_cols_norm<17>(cols);
                }
            }
            f9_cols_norm<17>(cols);
            red3[t] = f9_redc(cols);
            __builtin_amdgcn_sched_barrier(0);
        }
        F9 bi[3];
        beta_line_fold(a, b, m, vprev9, bi);
        // sums of at most 6 products below 128 r^2: the reduced values are normal and below 12 r
        const F9 ra = red3[0], rc = red3[1], rb = red3[2];
        if (a.ps_write)
            psum_store(a, b, f9_norm_reduce(ra), f9_norm_reduce(rc), f9_norm_reduce(f9_add(f9_add(rb, ra), rc)));
        // limbs of ra, rb, rc are below 2^29: at most eight of them are added between carry passes
        const F9 c2 = f9_add(rc, rc), c4 = f9_add(c2, c2), b2 = f9_add(rb, rb), a2 = f9_add(ra, ra);
        const F9 g2 = f9_norm(f9_add(f9_add(ra, c4), b2));                 // A' + 4 C' + 2 B
        const F9 t1 = f9_norm(f9_add(f9_add(a2, a2), c4));                 // 4 A' + 4 C'
        const F9 t2 = f9_norm(f9_add(f9_add(c4, rc), b2));                 // 5 C' + 2 B
        const F9 t3 = f9_norm(f9_add(b2, b2));                             // 4 B
        const F9 g3 = f9_norm(f9_add(f9_add(t1, t2), t3));                 // 4 A' + 9 C' + 6 B
        tot[0] = f9_norm_reduce(f9_add(tot[0], f9_mul(bi[0], ra)));
        tot[1] = f9_norm_reduce(f9_add(tot[1], f9_mul(bi[1], g2)));
        tot[2] = f9_norm_reduce(f9_add(tot[2], f9_mul(bi[2], g3)));
    }
    {
        const Fr s = block_sum_lazy<3>(tot, red);
        Fr* p = a.part + (uint64_t)bx * 4;
        if (tid < 3) p[tid ? tid + 1 : 0] = s;
        else if (tid == 3) p[1] = fr_zero();
    }
}

// After the second challenge: entry (k, v0, v1, i'', j) = A_lo + v1 (A_hi - A_lo), one of 16
// values by the four bits; written as lazy limbs, D/4 rows per column.
__global__ __launch_bounds__(ZK_BLOCK) void k_zk_mat2(BinArgs a) {
    __shared__ F9 val[16];
    if (threadIdx.x < 16) {
        const int c = threadIdx.x;
        const Fr v0 = a.chal[0], v1 = a.chal[1], one = fr_one();
        const Fr alo = bit_pair_value(c & 3, v0, one), ahi = bit_pair_value(c >> 2, v0, one);
        val[c] = fr_unpack(fr_add(alo, fr_mul(v1, fr_sub(ahi, alo))));
    }
    __syncthreads();
    const uint64_t m = a.m;   // rows written = D / 4
    int j0 = blockIdx.y * a.jc, j1 = j0 + a.jc;
    if (j1 > a.nbits) j1 = a.nbits;
    for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; b < m;
         b += (uint64_t)gridDim.x * blockDim.x) {
        for (int k = 0; k < (a.has_ga ? 2 : 1); ++k) {
            const int64_t* src = k == 0 ? a.z : a.ga;
            const uint64_t w00 = (uint64_t)src[b], w01 = (uint64_t)src[b + m];
            const uint64_t w10 = (uint64_t)src[b + 2 * m], w11 = (uint64_t)src[b + 3 * m];
            for (int j = j0; j < j1; ++j) {
                const int c = (int)((w00 >> j) & 1) | (int)(((w10 >> j) & 1) << 1) |
                              (int)(((w01 >> j) & 1) << 2) | (int)(((w11 >> j) & 1) << 3);
                f9tab_st(aux_col9(a, k, j), b, val[c]);
            }
        }
    }
}

// ---- round 2 by look-up as well -------------------------------------------------------
// With x0 = v0 and x1 = v1 bound an entry is one of the 16 values above, so the pair that
// round 2 interpolates is one of 256 combinations and q(x) = e(x)^2 - e(x) is a table of
// 256 entries per evaluation point, built once per block in LDS.  Per column that leaves
// a table read and the product with beta_J, accumulated as 64-bit columns.  The rows of
// pair index i3 (m = D/8 of them) are i3 + s m, s = 4 x0 + 2 x1 + x2.

// 16-value code of the entry at x2 from bit j of the eight rows (w[s] already shifted so
// that bit j is bit 0): bits (x0,x1) = (0,0), (1,0), (0,1), (1,1) as in k_zk_mat2
__device__ __forceinline__ uint32_t pair_code8(const uint64_t w[8]) {
    const uint32_t lo = ((uint32_t)w[0] & 1u) | (((uint32_t)w[4] & 1u) << 1) | (((uint32_t)w[2] & 1u) << 2) |
                        (((uint32_t)w[6] & 1u) << 3);
    const uint32_t hi = ((uint32_t)w[1] & 1u) | (((uint32_t)w[5] & 1u) << 1) | (((uint32_t)w[3] & 1u) << 2) |
                        (((uint32_t)w[7] & 1u) << 3);
    return lo | (hi << 4);
}

// the 16 values of an entry after v0, v1 (lazy limbs, normal, fully reduced)
__device__ __forceinline__ void bound2_values(const Fr* chal, F9* val16) {
    if (threadIdx.x < 16) {
        const int c = threadIdx.x;
        const Fr v0 = chal[0], v1 = chal[1], one = fr_one();
        const Fr alo = bit_pair_value(c & 3, v0, one), ahi = bit_pair_value(c >> 2, v0, one);
        val16[c] = fr_unpack(fr_add(alo, fr_mul(v1, fr_sub(ahi, alo))));
    }
}

template <bool PSUM>
__device__ __forceinline__ void bin2_body(const BinArgs& a, const unsigned bx, const unsigned by, const unsigned gx) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    __shared__ F9 sbj[2][64];
    __shared__ F9 val16[16];
    __shared__ uint32_t qlut[3][9][256];   // q(x) at x = 0, 2, 3 by combination, limb-major
    const int tid = threadIdx.x;
    if (tid < 128) {
        const int j = tid & 63, k = tid >> 6;
        F9 x = f9_zero();
        if (j < a.nbits) x = fr_unpack(k == 0 ? a.bJ[j] : fr_mul(*a.rp, a.bJ[j]));
        sbj[k][j] = x;
    }
    bound2_values(a.chal, val16);
    __syncthreads();
    {
        const F9 one9 = fr_unpack(fr_one());
        const F9 lo = val16[tid & 15], hi = val16[tid >> 4];
        const F9 dn = f9_norm(f9_sub(hi, lo));
        F9 e[3];
        e[0] = lo;
        e[1] = f9_norm(f9_add(hi, dn));
        e[2] = f9_norm(f9_add(e[1], dn));
        if (PSUM) {   // only (hi - lo)^2 is needed, kept in the first table
            const F9 q = f9_mul(dn, dn);
#pragma unroll
            for (int l = 0; l < 9; ++l) qlut[0][l][tid] = q.v[l];
        } else {
#pragma unroll
            for (int x = 0; x < 3; ++x) {
                const F9 q = f9_mul(e[x], f9_sub(e[x], one9));
#pragma unroll
                for (int l = 0; l < 9; ++l) qlut[x][l][tid] = q.v[l];
            }
        }
    }
    PsumConsts pk;
    if (PSUM) pk = psum_consts(a.vprev);
    __syncthreads();
    const uint64_t m = a.m;
    const F9 vprev9 = fr_unpack(*a.vprev);
    const unsigned chunk = a.ksplit ? by >> 1 : by;
    const int k0 = a.ksplit ? (int)(by & 1) : 0, k1 = a.ksplit ? k0 + 1 : (a.has_ga ? 2 : 1);
    int j0 = chunk * a.jc, j1 = j0 + a.jc;
    if (j1 > a.nbits) j1 = a.nbits;
    F9 tot[3];
#pragma unroll
    for (int x = 0; x < 3; ++x) tot[x] = f9_zero();
    for (uint64_t b = bx * (uint64_t)blockDim.x + tid; b < m; b += (uint64_t)gx * blockDim.x) {
        uint64_t cols[3][17];
#pragma unroll
        for (int x = 0; x < 3; ++x)
#pragma unroll
            for (int c = 0; c < 17; ++c) cols[x][c] = 0;
        int pending = 0;
        for (int k = k0; k < k1; ++k) {
            const int64_t* src = k == 0 ? a.z : a.ga;
            uint64_t w[8];
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2) w[s2] = (uint64_t)src[b + (uint64_t)s2 * m] >> j0;
            for (int j = j0; j < j1; ++j) {
                const uint32_t C = pair_code8(w);
#pragma unroll
                for (int s2 = 0; s2 < 8; ++s2) w[s2] >>= 1;
                const F9 bj = sbj[k][j];
#pragma unroll
                for (int x = 0; x < (PSUM ? 1 : 3); ++x) {
                    F9 q;
#pragma unroll
                    for (int l = 0; l < 9; ++l) q.v[l] = qlut[x][l][C];
                    f9_cols_mac(cols[x], bj, q);
                }
                if (++pending == 4) {
                    pending = 0;
#pragma unroll
                    for (int x = 0; x < (PSUM ? 1 : 3); ++x) f9_cols_norm<17>(cols[x]);
                }
            }
        }
        F9 bi[3];
        beta_line_fold(a, b, m, vprev9, bi);
        if (PSUM) {
            f9_cols_norm<17>(cols[0]);
            const F9 sd = f9_norm_reduce(f9_redc(cols[0]));
            F9 sa = f9_zero(), sc = f9_zero();
            if (chunk == 0 && k0 == 0) psum_bind(a, b, m, pk, sa, sc);
            if (a.ps_write) psum_store(a, (uint64_t)by * m + b, sa, sc, sd);
            psum_accumulate(tot, bi, sa, sc, sd);
        } else {
#pragma unroll
            for (int x = 0; x < 3; ++x) {
                f9_cols_norm<17>(cols[x]);
                tot[x] = f9_norm_reduce(f9_add(tot[x], f9_mul(bi[x], f9_redc(cols[x]))));
            }
        }
    }
    const uint64_t blk = (uint64_t)by * gx + bx;
    {
        const Fr s = block_sum_lazy<3>(tot, red);
        Fr* p = a.part + blk * 4;
        if (tid < 3) p[tid ? tid + 1 : 0] = s;
        else if (tid == 3) p[1] = fr_zero();
    }
}

// After the third challenge (8 <= D < 16 only; larger D write their columns after the fourth):
// entry (k, v0, v1, v2, i3, j) = lo + v2 (hi - lo), one of 256 values by the eight bits; written
// as lazy limbs, D/8 rows per column.
__global__ __launch_bounds__(ZK_BLOCK) void k_zk_mat3(BinArgs a) {
    __shared__ F9 val16[16];
    __shared__ uint32_t vlut[9][256];
    const int tid = threadIdx.x;
    bound2_values(a.chal, val16);
    __syncthreads();
    {
        const F9 v2 = fr_unpack(a.chal[2]);
        const F9 lo = val16[tid & 15], hi = val16[tid >> 4];
        const F9 f = f9_norm_reduce(f9_add(lo, f9_mul(f9_sub(hi, lo), v2)));
#pragma unroll
        for (int l = 0; l < 9; ++l) vlut[l][tid] = f.v[l];
    }
    __syncthreads();
    const uint64_t m = a.m;   // rows written = D / 8
    int j0 = blockIdx.y * a.jc, j1 = j0 + a.jc;
    if (j1 > a.nbits) j1 = a.nbits;
    for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + tid; b < m; b += (uint64_t)gridDim.x * blockDim.x) {
        for (int k = 0; k < (a.has_ga ? 2 : 1); ++k) {
            const int64_t* src = k == 0 ? a.z : a.ga;
            uint64_t w[8];
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2) w[s2] = (uint64_t)src[b + (uint64_t)s2 * m] >> j0;
            for (int j = j0; j < j1; ++j) {
                const uint32_t C = pair_code8(w);
#pragma unroll
                for (int s2 = 0; s2 < 8; ++s2) w[s2] >>= 1;
                F9 f;
#pragma unroll
                for (int l = 0; l < 9; ++l) f.v[l] = vlut[l][C];
                f9tab_st(aux_col9(a, k, j), b, f);
            }
        }
    }
}

// ---- round 3 from the integers; the columns are written after the fourth challenge -------
// With three challenges bound an entry is one of 256 values A[c] (c: its eight bits, as in
// k_zk_mat3).  Round 3 pairs two of them, 65 536 combinations: too many for a table of q(x), but
//   q(X) = e(X)^2 - e(X) = (1 - X) p(lo) + X p(hi) - X (1 - X) (hi - lo)^2,   p(a) = a^2 - a,
// and p(lo), p(hi) are table entries too (P[c] = A[c]^2 - A[c]): one square per column instead
// of three, and no column in memory yet.  Per pair index the sums over the columns
//   SA = sum beta_J p(lo), SC = sum beta_J p(hi), SD = sum beta_J (hi - lo)^2
// are accumulated as 64-bit columns; G(0) = SA, G(2) = -SA + 2 SC + 2 SD, G(3) = -2 SA + 3 SC + 6 SD.
// The rows of pair index i4 (m = D/16 of them) are i4 + s m, s = 8 x0 + 4 x1 + 2 x2 + x3.

// A[c] for the 256 codes: lazy limbs, normal, below 2.41 r; limb-major in LDS
__device__ __forceinline__ void bound3_values(const Fr* chal, F9* val16, uint32_t (*alut)[256]) {
    bound2_values(chal, val16);
    __syncthreads();
    const int tid = threadIdx.x;
    const F9 v2 = fr_unpack(chal[2]);
    const F9 lo = val16[tid & 15], hi = val16[tid >> 4];
    const F9 f = f9_norm_reduce(f9_add(lo, f9_mul(f9_sub(hi, lo), v2)));
#pragma unroll
    for (int l = 0; l < 9; ++l) alut[l][tid] = f.v[l];
}

__device__ __forceinline__ F9 lut9(const uint32_t (*lut)[256], uint32_t c) {
    F9 f;
#pragma unroll
    for (int l = 0; l < 9; ++l) f.v[l] = lut[l][c];
    return f;
}

// codes of the two entries that bit j of the sixteen rows w[s] gives: even rows (x3 = 0) and
// odd rows (x3 = 1), each in the bit order of pair_code8
__device__ __forceinline__ void pair_codes16(const uint64_t w[16], int j, uint32_t& clo, uint32_t& chi) {
    uint64_t e[8], o[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        e[s] = w[2 * s] >> j;
        o[s] = w[2 * s + 1] >> j;
    }
    clo = pair_code8(e);
    chi = pair_code8(o);
}

template <bool PSUM>
__device__ __forceinline__ void bin3_body(const BinArgs& a, const unsigned bx, const unsigned by, const unsigned gx) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    __shared__ F9 sbj[2][64];
    __shared__ F9 val16[16];
    __shared__ uint32_t alut[9][256];   // A[c]
    __shared__ uint32_t plut[9][256];   // A[c]^2 - A[c]
    const int tid = threadIdx.x;
    if (tid < 128) {
        const int j = tid & 63, k = tid >> 6;
        F9 x = f9_zero();
        if (j < a.nbits) x = fr_unpack(k == 0 ? a.bJ[j] : fr_mul(*a.rp, a.bJ[j]));
        sbj[k][j] = x;
    }
    bound3_values(a.chal, val16, alut);
    PsumConsts pk;
    if (PSUM) pk = psum_consts(a.vprev);
    if (!PSUM) {
        const F9 one9 = fr_unpack(fr_one());
        const F9 f = lut9(alut, tid);
        const F9 q = f9_mul(f, f9_sub(f, one9));      // normal, below 2 r
#pragma unroll
        for (int l = 0; l < 9; ++l) plut[l][tid] = q.v[l];
    }
    __syncthreads();
    const uint64_t m = a.m;
    const F9 vprev9 = fr_unpack(*a.vprev);
    const unsigned chunk = a.ksplit ? by >> 1 : by;
    const int k0 = a.ksplit ? (int)(by & 1) : 0, k1 = a.ksplit ? k0 + 1 : (a.has_ga ? 2 : 1);
    int j0 = chunk * a.jc, j1 = j0 + a.jc;
    if (j1 > a.nbits) j1 = a.nbits;
    F9 tot[3];
#pragma unroll
    for (int x = 0; x < 3; ++x) tot[x] = f9_zero();
    for (uint64_t b = bx * (uint64_t)blockDim.x + tid; b < m; b += (uint64_t)gx * blockDim.x) {
        uint64_t cols[3][17];   // SA, SC, SD
#pragma unroll
        for (int x = 0; x < 3; ++x)
#pragma unroll
            for (int c = 0; c < 17; ++c) cols[x][c] = 0;
        int pending = 0;
        for (int k = k0; k < k1; ++k) {
            const int64_t* src = k == 0 ? a.z : a.ga;
            uint64_t w[16];
#pragma unroll
            for (int s2 = 0; s2 < 16; ++s2) w[s2] = (uint64_t)src[b + (uint64_t)s2 * m];
            for (int j = j0; j < j1; ++j) {
                uint32_t clo, chi;
                pair_codes16(w, j, clo, chi);
                const F9 bj = sbj[k][j];
                if (!PSUM) {
                    f9_cols_mac(cols[0], bj, lut9(plut, clo));
                    f9_cols_mac(cols[1], bj, lut9(plut, chi));
                }
                const F9 d = f9_norm(f9_sub(lut9(alut, chi), lut9(alut, clo)));   // normal, below 6.5 r
                f9_cols_mac(cols[2], bj, f9_mul(d, d));
                if (++pending == 4) {
                    pending = 0;
#pragma unroll
                    for (int x = (PSUM ? 2 : 0); x < 3; ++x) f9_cols_norm<17>(cols[x]);
                }
            }
        }
        F9 bi[3];
        beta_line_fold(a, b, m, vprev9, bi);
#pragma unroll
        for (int x = (PSUM ? 2 : 0); x < 3; ++x) f9_cols_norm<17>(cols[x]);
        // at most 128 products below 2 r^2 each: the reduced sums are below 4.8 r before the reducing pass
        F9 sa, sc;
        const F9 sd = f9_norm_reduce(f9_redc(cols[2]));
        if (PSUM) {
            sa = f9_zero();
            sc = f9_zero();
            if (chunk == 0 && k0 == 0) psum_bind(a, b, m, pk, sa, sc);
        } else {
            sa = f9_norm_reduce(f9_redc(cols[0]));
            sc = f9_norm_reduce(f9_redc(cols[1]));
        }
        if (a.ps_write) psum_store(a, (uint64_t)by * m + b, sa, sc, sd);
        psum_accumulate(tot, bi, sa, sc, sd);
    }
    const uint64_t blk = (uint64_t)by * gx + bx;
    {
        const Fr s = block_sum_lazy<3>(tot, red);
        Fr* p = a.part + blk * 4;
        if (tid < 3) p[tid ? tid + 1 : 0] = s;
        else if (tid == 3) p[1] = fr_zero();
    }
}

// After the fourth challenge: entry (k, v0..v3, i4, j) = (1 - v3) A[c_lo] + v3 A[c_hi]: two table
// reads and an addition; written as lazy limbs (normal, below 2 r), D/16 rows per column.
__global__ __launch_bounds__(ZK_BLOCK) void k_zk_mat4(BinArgs a) {
    __shared__ F9 val16[16];
    __shared__ uint32_t alut[9][256];
    __shared__ uint32_t lut0[9][256];   // (1 - v3) A[c], fully reduced
    __shared__ uint32_t lut1[9][256];   // v3 A[c], fully reduced
    const int tid = threadIdx.x;
    bound3_values(a.chal, val16, alut);
    {
        const Fr v3 = a.chal[3], u3 = fr_sub(fr_one(), v3);
        const F9 f = lut9(alut, tid);
        const F9 f0 = f9_cond_sub(f9_mul(fr_unpack(u3), f)), f1 = f9_cond_sub(f9_mul(fr_unpack(v3), f));
#pragma unroll
        for (int l = 0; l < 9; ++l) {
            lut0[l][tid] = f0.v[l];
            lut1[l][tid] = f1.v[l];
        }
    }
    __syncthreads();
    const uint64_t m = a.m;   // rows written = D / 16
    int j0 = blockIdx.y * a.jc, j1 = j0 + a.jc;
    if (j1 > a.nbits) j1 = a.nbits;
    for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + tid; b < m; b += (uint64_t)gridDim.x * blockDim.x) {
        for (int k = 0; k < (a.has_ga ? 2 : 1); ++k) {
            const int64_t* src = k == 0 ? a.z : a.ga;
            uint64_t w[16];
#pragma unroll
            for (int s2 = 0; s2 < 16; ++s2) w[s2] = (uint64_t)src[b + (uint64_t)s2 * m];
            for (int j = j0; j < j1; ++j) {
                uint32_t clo, chi;
                pair_codes16(w, j, clo, chi);
                f9tab_st(aux_col9(a, k, j), b, f9_norm(f9_add(lut9(lut0, clo), lut9(lut1, chi))));
            }
        }
    }
}

// ---- round 4 from the integers; the columns are written after the fifth challenge ----------
// Taken when the column sums reach round 4 and its columns are not cut into chunks (large D): the
// round then needs only sum_j beta_J (hi_j - lo_j)^2, and an entry with four challenges bound is
// (1 - v3) A[c_lo] + v3 A[c_hi] by the 16 bits it interpolates (as in k_zk_mat4), so nothing has to
// be in memory yet and the columns are written with half the rows once more.  The rows of pair
// index i5 (m = D/32 of them) are i5 + s m, s = 16 x0 + 8 x1 + 4 x2 + 2 x3 + x4.  Bit j of all 32
// rows is wanted for every column j: the 32 x 64 bit matrix of the rows is transposed once (two
// 32 x 32 blocks, five swap stages each), with the rows ordered so that the four codes of a
// column are the four bytes of its word.

// in-place transpose of a 32 x 32 bit matrix: afterwards bit p of a[j] is what bit j of a[p] was
__device__ __forceinline__ void transpose32(uint32_t a[32]) {
#pragma unroll
    for (int s = 0; s < 5; ++s) {
        const int j = 16 >> s;
        const uint32_t m = s == 0 ? 0x0000FFFFu : s == 1 ? 0x00FF00FFu : s == 2 ? 0x0F0F0F0Fu : s == 3 ? 0x33333333u : 0x55555555u;
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            if (k & j) continue;
            const uint32_t t = ((a[k] >> j) ^ a[k + j]) & m;
            a[k] ^= t << j;
            a[k + j] ^= t;
        }
    }
}

// Row that lands in bit p of a column's word: byte g = 2 x4 + x3 holds the code (bit order of
// pair_code8) of the eight rows with that (x3, x4).
__device__ __forceinline__ int bin4_row_of_bit(int p) {
    const int order8[8] = {0, 4, 2, 6, 1, 5, 3, 7};
    const int g = p >> 3, q = p & 7;
    return 4 * order8[q] + 2 * (g & 1) + (g >> 1);
}

// words of 32 columns (bit p = bit j of row bin4_row_of_bit(p)), columns 32 half .. 32 half + 31,
// left in the thread's own slots cw[.][threadIdx.x]: the column loop then runs over j without
// being unrolled (no barrier is needed, no thread reads another's slots)
__device__ __forceinline__ void bin4_columns(const int64_t* src, uint64_t b, uint64_t m, int half, uint32_t (*cw)[ZK_BLOCK]) {
    uint32_t a32[32];
#pragma unroll
    for (int p = 0; p < 32; ++p) {
        const uint64_t w = (uint64_t)src[b + (uint64_t)bin4_row_of_bit(p) * m];
        a32[p] = half ? (uint32_t)(w >> 32) : (uint32_t)w;
    }
    transpose32(a32);
#pragma unroll
    for (int p = 0; p < 32; ++p) cw[p][threadIdx.x] = a32[p];
}

struct Bin4Luts {
    uint32_t lut0[9][256];   // (1 - v3) A[c], fully reduced; A[c]: the entry with three challenges bound
    uint32_t lut1[9][256];   // v3 A[c], fully reduced
};

// scratch: 9 x 256 words that are free until the tables are built (all threads; ends with a barrier)
__device__ __forceinline__ void bin4_luts_build(const Fr* chal, F9* val16, uint32_t (*scratch)[256], Bin4Luts& L) {
    bound3_values(chal, val16, scratch);
    const int tid = threadIdx.x;
    const Fr v3 = chal[3], u3 = fr_sub(fr_one(), v3);
    const F9 f = lut9(scratch, tid);     // the thread's own entry
    const F9 f0 = f9_cond_sub(f9_mul(fr_unpack(u3), f)), f1 = f9_cond_sub(f9_mul(fr_unpack(v3), f));
#pragma unroll
    for (int l = 0; l < 9; ++l) {
        L.lut0[l][tid] = f0.v[l];
        L.lut1[l][tid] = f1.v[l];
    }
    __syncthreads();
}

__device__ __forceinline__ void bin4_body(const BinArgs& a, const unsigned bx, const unsigned gx) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    __shared__ F9 sbj[2][64];
    __shared__ F9 val16[16];
    __shared__ Bin4Luts L;
    __shared__ uint32_t cw[32][ZK_BLOCK];   // a thread's column words, 32 columns at a time
    const int tid = threadIdx.x;
    if (tid < 128) {
        const int j = tid & 63, k = tid >> 6;
        F9 x = f9_zero();
        if (j < a.nbits) x = fr_unpack(k == 0 ? a.bJ[j] : fr_mul(*a.rp, a.bJ[j]));
        sbj[k][j] = x;
    }
    bin4_luts_build(a.chal, val16, (uint32_t (*)[256])&cw[0][0], L);
    const PsumConsts pk = psum_consts(a.vprev);
    const uint64_t m = a.m;
    F9 tot[3];
#pragma unroll
    for (int x = 0; x < 3; ++x) tot[x] = f9_zero();
    for (uint64_t b = bx * (uint64_t)blockDim.x + tid; b < m; b += (uint64_t)gx * blockDim.x) {
        uint64_t cols[17];
#pragma unroll
        for (int c = 0; c < 17; ++c) cols[c] = 0;
        int pending = 0;
        for (int k = 0; k < (a.has_ga ? 2 : 1); ++k) {
            for (int half = 0; 32 * half < a.nbits; ++half) {
                bin4_columns(k == 0 ? a.z : a.ga, b, m, half, cw);
                const int jn = a.nbits - 32 * half < 32 ? a.nbits - 32 * half : 32;
                for (int jj = 0; jj < jn; ++jj) {
                    const uint32_t w = cw[jj][tid];
                    // entries at x4 = 0 (bytes 0, 1) and x4 = 1 (bytes 2, 3), each below 2 r
                    const F9 e0 = f9_norm(f9_add(lut9(L.lut0, w & 255), lut9(L.lut1, (w >> 8) & 255)));
                    const F9 e1 = f9_add(lut9(L.lut0, (w >> 16) & 255), lut9(L.lut1, w >> 24));
                    const F9 d = f9_norm(f9_sub(e1, e0));     // limbs of e1 below 2^30; normal, below 6 r
                    f9_cols_mac(cols, sbj[k][32 * half + jj], f9_mul(d, d));
                    if (++pending == 4) {
                        pending = 0;
                        f9_cols_norm<17>(cols);
                    }
                }
            }
        }
        f9_cols_norm<17>(cols);
        const F9 sd = f9_norm_reduce(f9_redc(cols));
        F9 sa, sc;
        psum_bind(a, b, m, pk, sa, sc);
        if (a.ps_write) psum_store(a, b, sa, sc, sd);
        F9 bi[3];
        beta_line_fold(a, b, m, pk.v, bi);
        psum_accumulate(tot, bi, sa, sc, sd);
    }
    {
        const Fr s = block_sum_lazy<3>(tot, red);
        Fr* p = a.part + (uint64_t)bx * 4;
        if (tid < 3) p[tid ? tid + 1 : 0] = s;
        else if (tid == 3) p[1] = fr_zero();
    }
}

// After the fifth challenge: entry (k, v0..v4, i5, j) = (1 - v4) e0 + v4 e1 with e0, e1 as in
// bin4_body: four table reads and three additions; lazy limbs (normal, below 2.41 r), D/32 rows.
__global__ __launch_bounds__(ZK_BLOCK) void k_zk_mat5(BinArgs a) {
    __shared__ F9 val16[16];
    __shared__ uint32_t t4[4][9][256];   // (1-v4)(1-v3) A, (1-v4) v3 A, v4 (1-v3) A, v4 v3 A; fully reduced
    __shared__ uint32_t cw[32][ZK_BLOCK];
    const int tid = threadIdx.x;
    {
        uint32_t (*alut)[256] = (uint32_t (*)[256])&cw[0][0];   // free until the first columns are transposed
        bound3_values(a.chal, val16, alut);
        const Fr v3 = a.chal[3], u3 = fr_sub(fr_one(), v3), v4 = a.chal[4], u4 = fr_sub(fr_one(), v4);
        const F9 f = lut9(alut, tid);   // the thread's own entry
        const Fr c[4] = {fr_mul(u4, u3), fr_mul(u4, v3), fr_mul(v4, u3), fr_mul(v4, v3)};
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const F9 q = f9_cond_sub(f9_mul(fr_unpack(c[g]), f));
#pragma unroll
            for (int l = 0; l < 9; ++l) t4[g][l][tid] = q.v[l];
        }
    }
    __syncthreads();
    const uint64_t m = a.m;   // rows written = D / 32
    for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + tid; b < m; b += (uint64_t)gridDim.x * blockDim.x) {
        for (int k = 0; k < (a.has_ga ? 2 : 1); ++k) {
            for (int half = 0; 32 * half < a.nbits; ++half) {
                bin4_columns(k == 0 ? a.z : a.ga, b, m, half, cw);
                const int jn = a.nbits - 32 * half < 32 ? a.nbits - 32 * half : 32;
                for (int jj = 0; jj < jn; ++jj) {
                    const uint32_t w = cw[jj][tid];
                    const F9 e = f9_add(f9_add(lut9(t4[0], w & 255), lut9(t4[1], (w >> 8) & 255)),
                                        f9_add(lut9(t4[2], (w >> 16) & 255), lut9(t4[3], w >> 24)));
                    f9tab_st(aux_col9(a, k, 32 * half + jj), b, f9_norm_reduce(e));
                }
            }
        }
    }
}

// the raw entries of one column that a pair index needs: (b, b+m), or (b, b+m, b+2m, b+3m)
// when the previous challenge is still to be bound
template <bool FOLD>
struct ColRaw {
    F9 t[FOLD ? 4 : 2];
};

template <bool FOLD>
__device__ __forceinline__ ColRaw<FOLD> col_load(const BinArgs& a, int k, int j, uint64_t b, uint64_t m) {
    const F9Tab col = aux_col9(a, k, j);
    ColRaw<FOLD> r;
#pragma unroll
    for (int q = 0; q < (FOLD ? 4 : 2); ++q) r.t[q] = f9tab_ld(col, b + (uint64_t)q * m);
    return r;
}

// Rounds after the materialisation, on the columns in memory (lazy limbs, same invariants as the product
// round kernel): per (i', j, slice) the pair (lo, hi), folded with the previous challenge
// first when FOLD; q(x) = e(x) (e(x) - 1) at x = 0, 2, 3; per thread the sum over its columns
// of beta_J(j) q(x) (slice 1 with r' beta_J), then times beta_I(x, i').
template <bool FOLD>
__device__ __forceinline__ void binl_body(const BinArgs& a, const unsigned bx, const unsigned by, const unsigned gx) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    __shared__ F9 sbj[2][64];
    const int tid = threadIdx.x;
    if (tid < 128) {
        const int j = tid & 63, k = tid >> 6;
        F9 x = f9_zero();
        if (j < a.nbits) x = fr_unpack(k == 0 ? a.bJ[j] : fr_mul(*a.rp, a.bJ[j]));
        sbj[k][j] = x;
    }
    __syncthreads();
    const uint64_t m = a.m;
    const F9 vprev9 = fr_unpack(*a.vprev);
    F9 v = f9_zero();
    if (FOLD) v = fr_unpack(*a.chal);
    const F9 one9 = fr_unpack(fr_one());
    const unsigned chunk = a.ksplit ? by >> 1 : by;
    const int k0 = a.ksplit ? (int)(by & 1) : 0, k1 = a.ksplit ? k0 + 1 : (a.has_ga ? 2 : 1);
    int j0 = chunk * a.jc, j1 = j0 + a.jc;
    if (j1 > a.nbits) j1 = a.nbits;
    // per-thread sums over the pair indices live in LDS: the column loop needs every register
    __shared__ uint32_t tot_s[3][9][ZK_BLOCK];
#pragma unroll
    for (int x = 0; x < 3; ++x)
#pragma unroll
        for (int l = 0; l < 9; ++l) tot_s[x][l][tid] = 0;
    for (uint64_t b = bx * (uint64_t)blockDim.x + tid; b < m; b += (uint64_t)gx * blockDim.x) {
        // sum over the columns of beta_J(j) q(x) as 64-bit columns: one reduction per (i', x)
        uint64_t cols[3][17];
#pragma unroll
        for (int x = 0; x < 3; ++x)
#pragma unroll
            for (int c = 0; c < 17; ++c) cols[x][c] = 0;
        int pending = 0;
        // the raw entries of the next column are requested before the current one is worked on
        const int nk = k1 - k0, ncol = (j1 - j0) * nk;
        ColRaw<FOLD> cur = col_load<FOLD>(a, k0, j0, b, m);
        for (int c = 0; c < ncol; ++c) {
            const int j = j0 + (nk == 2 ? c >> 1 : c), k = k0 + (nk == 2 ? (c & 1) : 0);
            const int cn = c + 1 < ncol ? c + 1 : c;   // the last iteration asks for its own column again
            const ColRaw<FOLD> nxt =
                col_load<FOLD>(a, k0 + (nk == 2 ? (cn & 1) : 0), j0 + (nk == 2 ? cn >> 1 : cn), b, m);
            F9 lo, hi;
            if (FOLD) {
                const F9Tab col = aux_col9(a, k, j);
                lo = f9_norm_reduce(f9_add(cur.t[0], f9_mul(f9_sub(cur.t[2], cur.t[0]), v)));
                hi = f9_norm_reduce(f9_add(cur.t[1], f9_mul(f9_sub(cur.t[3], cur.t[1]), v)));
                f9tab_st(col, b, lo);
                f9tab_st(col, b + m, hi);
            } else {
                lo = cur.t[0];
                hi = cur.t[1];
            }
            const F9 bj = sbj[k][j];
            const F9 dn = f9_norm(f9_sub(hi, lo));
            // e (e - 1) at x = 0, 2, 3: e normal, e - 1 + 4r has limbs < 2^29 + 2^30; the product is normal
            F9 e = lo;
            f9_cols_mac(cols[0], bj, f9_mul(e, f9_sub(e, one9)));
            e = f9_norm(f9_add(hi, dn));
            f9_cols_mac(cols[1], bj, f9_mul(e, f9_sub(e, one9)));
            e = f9_norm(f9_add(e, dn));
            f9_cols_mac(cols[2], bj, f9_mul(e, f9_sub(e, one9)));
            if (++pending == 4) {
                pending = 0;
#pragma unroll
                for (int x = 0; x < 3; ++x) f9_cols_norm<17>(cols[x]);
            }
            cur = nxt;
        }
        F9 bi[3];
        beta_line_fold(a, b, m, vprev9, bi);
#pragma unroll
        for (int x = 0; x < 3; ++x) {
            // at most 128 products below 2 r^2 each: the reduced sum is below 4.8 r, normal
            f9_cols_norm<17>(cols[x]);
            F9 t;
#pragma unroll
            for (int l = 0; l < 9; ++l) t.v[l] = tot_s[x][l][tid];
            t = f9_norm_reduce(f9_add(t, f9_mul(bi[x], f9_redc(cols[x]))));
#pragma unroll
            for (int l = 0; l < 9; ++l) tot_s[x][l][tid] = t.v[l];
        }
    }
    const uint64_t blk = (uint64_t)by * gx + bx;
    {
        F9 tot[3];
#pragma unroll
        for (int x = 0; x < 3; ++x)
#pragma unroll
            for (int l = 0; l < 9; ++l) tot[x].v[l] = tot_s[x][l][tid];
        const Fr s = block_sum_lazy<3>(tot, red);
        Fr* p = a.part + blk * 4;
        if (tid < 3) p[tid ? tid + 1 : 0] = s;
        else if (tid == 3) p[1] = fr_zero();
    }
}

// The same rounds when the previous round left its column sums (psum_bind): only
// SD' = sum_j beta_J (hi'_j - lo'_j)^2 needs the columns, one square per column instead of three and
// one accumulator instead of three.  With the columns cut into chunks, the thread of the first
// chunk (and slice) takes SA' and SC'.
template <bool FOLD>
__device__ __forceinline__ void binp_body(const BinArgs& a, const unsigned bx, const unsigned by, const unsigned gx) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    __shared__ F9 sbj[2][64];
    const int tid = threadIdx.x;
    if (tid < 128) {
        const int j = tid & 63, k = tid >> 6;
        F9 x = f9_zero();
        if (j < a.nbits) x = fr_unpack(k == 0 ? a.bJ[j] : fr_mul(*a.rp, a.bJ[j]));
        sbj[k][j] = x;
    }
    __syncthreads();
    const uint64_t m = a.m;
    const PsumConsts pk = psum_consts(a.vprev);
    const F9 v = pk.v;                    // the challenge that this round binds on the way
    const unsigned chunk = a.ksplit ? by >> 1 : by;
    const int k0 = a.ksplit ? (int)(by & 1) : 0, k1 = a.ksplit ? k0 + 1 : (a.has_ga ? 2 : 1);
    int j0 = chunk * a.jc, j1 = j0 + a.jc;
    if (j1 > a.nbits) j1 = a.nbits;
    F9 tot[3];
#pragma unroll
    for (int x = 0; x < 3; ++x) tot[x] = f9_zero();
    for (uint64_t b = bx * (uint64_t)blockDim.x + tid; b < m; b += (uint64_t)gx * blockDim.x) {
        uint64_t cols[17];
#pragma unroll
        for (int c = 0; c < 17; ++c) cols[c] = 0;
        int pending = 0;
        const int nk = k1 - k0, ncol = (j1 - j0) * nk;
        ColRaw<FOLD> cur = col_load<FOLD>(a, k0, j0, b, m);
        for (int c = 0; c < ncol; ++c) {
            const int j = j0 + (nk == 2 ? c >> 1 : c), k = k0 + (nk == 2 ? (c & 1) : 0);
            const int cn = c + 1 < ncol ? c + 1 : c;   // the last iteration asks for its own column again
            const ColRaw<FOLD> nxt =
                col_load<FOLD>(a, k0 + (nk == 2 ? (cn & 1) : 0), j0 + (nk == 2 ? cn >> 1 : cn), b, m);
            F9 lo, hi;
            if (FOLD) {
                const F9Tab col = aux_col9(a, k, j);
                lo = f9_norm_reduce(f9_add(cur.t[0], f9_mul(f9_sub(cur.t[2], cur.t[0]), v)));
                hi = f9_norm_reduce(f9_add(cur.t[1], f9_mul(f9_sub(cur.t[3], cur.t[1]), v)));
                f9tab_st(col, b, lo);
                f9tab_st(col, b + m, hi);
            } else {
                lo = cur.t[0];
                hi = cur.t[1];
            }
            const F9 d = f9_norm(f9_sub(hi, lo));     // normal, below 6.5 r
            f9_cols_mac(cols, sbj[k][j], f9_mul(d, d));
            if (++pending == 4) {
                pending = 0;
                f9_cols_norm<17>(cols);
            }
            cur = nxt;
        }
        f9_cols_norm<17>(cols);
        const F9 sd = f9_norm_reduce(f9_redc(cols));   // at most 128 products below 2 r^2: below 4.8 r before
        F9 sa = f9_zero(), sc = f9_zero();
        if (chunk == 0 && k0 == 0) psum_bind(a, b, m, pk, sa, sc);
        if (a.ps_write) psum_store(a, (uint64_t)by * m + b, sa, sc, sd);
        F9 bi[3];
        beta_line_fold(a, b, m, v, bi);
        psum_accumulate(tot, bi, sa, sc, sd);
    }
    const uint64_t blk = (uint64_t)by * gx + bx;
    {
        const Fr s = block_sum_lazy<3>(tot, red);
        Fr* p = a.part + blk * 4;
        if (tid < 3) p[tid ? tid + 1 : 0] = s;
        else if (tid == 3) p[1] = fr_zero();
    }
}

// One launch per i-round: the first nb_lin blocks take the linear equations, the others the
// binarity terms (column chunk = block / bin_gx).  The two parts share no table, so they run
// side by side; their partial sums land in one array that the round's finaliser adds up.
struct ZkRoundArgs {
    LinArgs lin;
    BinArgs bin;
    unsigned nb_lin, bin_gx;
    int lin_small;         // the linear blocks take LIN_SMALL_PAIRS pairs each
};

// MODE 0: first round; 1, 2, 5: rounds 1, 2, 3 on the integers; 3: first round on the columns
// in memory; 4: later rounds (fold the columns with the previous challenge first); 6, 7, 8, 9: as 3,
// 4, 2, 5 with the column sums of the previous round at hand; 10: round 4 on the integers (with them)
template <int MODE>
__global__ __launch_bounds__(ZK_BLOCK, 2) void k_zk_round(ZkRoundArgs a) {
    if (blockIdx.x < a.nb_lin) {
        if (MODE <= 1 && a.lin.from_ints) {
            if (MODE == 0) lin0_int_body(a.lin, blockIdx.x);
            else lin1_int_body(a.lin, blockIdx.x);
        } else if (MODE >= 2 && a.lin.split_eq) lin_body<true, true>(a.lin, blockIdx.x, a.nb_lin);
        else if (a.lin_small) lin_body_small<MODE != 0>(a.lin, blockIdx.x);
        else lin_body<MODE != 0, false>(a.lin, blockIdx.x, a.nb_lin);
        return;
    }
    const unsigned bid = blockIdx.x - a.nb_lin;
    const unsigned bx = bid % a.bin_gx, by = bid / a.bin_gx;
    if (MODE == 0) bin0_body(a.bin, bx, a.bin_gx);
    else if (MODE == 1) bin1_body(a.bin, bx, a.bin_gx);
    else if (MODE == 2 || MODE == 8) bin2_body<MODE == 8>(a.bin, bx, by, a.bin_gx);
    else if (MODE == 5 || MODE == 9) bin3_body<MODE == 9>(a.bin, bx, by, a.bin_gx);
    else if (MODE == 6 || MODE == 7) binp_body<MODE == 7>(a.bin, bx, by, a.bin_gx);
    else if (MODE == 10) bin4_body(a.bin, bx, a.bin_gx);
    else binl_body<MODE == 4>(a.bin, bx, by, a.bin_gx);
}

template <int MODE>
static void launch_zk_round(zkdl_ctx* ctx, const ZkRoundArgs& ra, unsigned nb_bin) {
    hipLaunchKernelGGL((k_zk_round<MODE>), dim3(ra.nb_lin + nb_bin), dim3(ZK_BLOCK), 0, ctx->stream, ra);
}

// ---------------------------------------------------------------------------
// tail: last fold of the i-tables, the j-rounds, finals, merge
// ---------------------------------------------------------------------------
struct TailArgs {
    ZkTabs tabs;
    BinArgs bin;          // aux planes, z/ga, bJ
    int li, lj, q_bits, r_bits;
    int mat_bound;        // i-challenges bound when the aux columns were written (2 or 3)
    DevState* st;
    int chal_v;           // index of the first round challenge (i-rounds, then j-rounds)
    int chal_rho;         // rho0..2, then the merge challenges
    uint32_t rounds_off;  // g's of the combined sumcheck (all rounds)
    uint32_t finals_off;
    uint32_t merge_claim_off, merge_rounds_off, merge_finals_off;
};

constexpr int TAIL_THREADS = 256;

// sum over the 64 lanes of a wave; every lane of the wave must call; lane 0 holds the result
__device__ __forceinline__ Fr wave_sum_fr(Fr x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        Fr y;
#pragma unroll
        for (int l = 0; l < 8; ++l) y.v[l] = __shfl_down(x.v[l], off, 64);
        x = fr_add(x, y);
    }
    return x;
}

// The end of the combined sumcheck in one block: the i-tables at the full i-point, the
// log2 J rounds over j, the finals, and the merge of the three claims on aux.
//
// With every i bound, the summand over j is
//   a0 [L0 + B0 (a0 - 1)] + a1 [L1 + B1 (a1 - 1)],
//   L0 = r^2 beta_Z(v) s + r beta_A(v)(1-sign(v)) s',   B0 = beta_I(v) beta_J,
//   L1, B1 the same for slice 1 (with r'), a_k = aux~(k, v, j):
// six tables of J entries.  Work is spread as (evaluation point, slice, j): wave w takes the
// point x in {0, 2, 3}[w] and sums it by itself, so a round needs no cross-wave reduction.
__global__ __launch_bounds__(TAIL_THREADS) void k_zk_tail(TailArgs a) {
    __shared__ TsShared TS;
    __shared__ Fr T6[6][64];                               // A0, A1, L0, L1, B0, B1 over j
    __shared__ Fr S[64], SP[64];
    __shared__ Fr M[128], E[128];                          // merge tables over (k, j)
    __shared__ Fr sc[LIN_TABLES];
    __shared__ Fr g[4];
    __shared__ Fr fin[3];
    __shared__ Fr rho[3];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    DevState* st = a.st;
    block_ts_load(TS, st);
    if (wave == 3) wave_resolve_claim(st);   // the last i-round may still owe its claim; read after barriers
    const int J = 1 << a.lj, nbits = a.q_bits + a.r_bits;
    const Fr one = fr_one();
    Fr vlast = fr_zero();
    if (a.li >= 1) vlast = st->chal[a.chal_v + a.li - 1];

    // scalars: the D-sized tables at the full i-point
    if (tid < LIN_TABLES) {
        bool present = a.bin.has_ga || !(tid == T_BGA || tid == T_GA || tid == T_BGZ || tid == T_GAP);
        Fr lo = fr_zero();
        if (present) {
            lo = f9_to_fr(f9tab_ld(a.tabs.t[tid], 0));
            if (a.li >= 1) {
                Fr hi = f9_to_fr(f9tab_ld(a.tabs.t[tid], 1));
                lo = fr_add(lo, fr_mul_ni(vlast, fr_sub(hi, lo)));
            }
        }
        sc[tid] = lo;
    } else if (tid >= 64 && tid < 192) {
        // aux~(k, v, j) for k = wave - 1
        const int j = lane, k = wave - 1;
        Fr val = fr_zero();
        if (j < nbits && (k == 0 || a.bin.has_ga)) {
            const int64_t* src = k == 0 ? a.bin.z : a.bin.ga;
            if (a.li == 0) {
                val = (((uint64_t)src[0] >> j) & 1) ? one : fr_zero();
            } else if (a.li == 1) {
                // one challenge: the entry interpolates the bits of the two integers
                const int code = (int)(((uint64_t)src[0] >> j) & 1) | (int)((((uint64_t)src[1] >> j) & 1) << 1);
                val = bit_pair_value(code, vlast, one);
            } else {
                // the columns were written with mat_bound challenges bound; later rounds
                // folded them down to two rows
                F9Tab col = aux_col9(a.bin, k, j);
                val = f9_to_fr(f9tab_ld(col, 0));
                if (a.li > a.mat_bound) {
                    Fr hi = f9_to_fr(f9tab_ld(col, 1));
                    val = fr_add(val, fr_mul_ni(vlast, fr_sub(hi, val)));
                }
            }
        }
        T6[k][j] = val;
        M[64 * k + j] = val;
    } else if (tid >= 192) {
        // s_{Q+R}(j) and s'(j) (Sec. 3.1, App. A)
        const int j = lane;
        Fr s = fr_zero(), sp = fr_zero();
        if (j < nbits) {
            if (j < nbits - 1) s = fr_from_i64((int64_t)1 << j);
            else s = fr_from_i64(j == 63 ? INT64_MIN : -((int64_t)1 << j));
            if (j == a.r_bits - 1) sp = one;
            else if (j >= a.r_bits && j < nbits - 1) sp = fr_from_i64((int64_t)1 << (j - a.r_bits));
            else if (j == nbits - 1) sp = fr_from_i64(-((int64_t)1 << (a.q_bits - 1)));
        }
        S[j] = s;
        SP[j] = sp;
    }
    __syncthreads();
    {
        // L0, L1, B0, B1: one table per wave
        const int j = lane;
        const Fr ns = sc[T_NS];
        Fr val = fr_zero();
        if (j < J) {
            if (wave == 0) val = fr_add(fr_mul_ni(sc[T_BZ], S[j]), fr_mul_ni(fr_mul_ni(sc[T_BA], ns), SP[j]));
            else if (wave == 1) val = fr_add(fr_mul_ni(sc[T_BGA], S[j]), fr_mul_ni(fr_mul_ni(sc[T_BGZ], ns), SP[j]));
            else if (wave == 2) val = fr_mul_ni(sc[T_BI], a.bin.bJ[j]);
            else val = fr_mul_ni(fr_mul_ni(st->weights[4], sc[T_BI]), a.bin.bJ[j]);
        }
        T6[2 + wave][j] = val;
    }
    __syncthreads();

    int cur = J;
    for (int t = 0; t < a.lj; ++t) {
        const int half = cur >> 1;
        // wave w < 3: point x = 0, 2, 3; lane = (slice << 5) | j
        Fr f = fr_zero();
        const int k = lane >> 5, j = lane & 31;
        if (wave < 3 && j < half) {
            Fr av, lv, bv;
            {
                const Fr lo = T6[k][j], hi = T6[k][j + half];
                const Fr lL = T6[2 + k][j], hL = T6[2 + k][j + half];
                const Fr lB = T6[4 + k][j], hB = T6[4 + k][j + half];
                if (wave == 0) {
                    av = lo; lv = lL; bv = lB;
                } else {
                    const Fr da = fr_sub(hi, lo), dL = fr_sub(hL, lL), dB = fr_sub(hB, lB);
                    av = fr_add(hi, da); lv = fr_add(hL, dL); bv = fr_add(hB, dB);
                    if (wave == 2) {
                        av = fr_add(av, da); lv = fr_add(lv, dL); bv = fr_add(bv, dB);
                    }
                }
            }
            f = fr_mul_ni(av, fr_add(lv, fr_mul_ni(bv, fr_sub(av, one))));
        }
        if (wave < 3) {
            f = wave_sum_fr(f);
            if (lane == 0) g[wave == 0 ? 0 : wave + 1] = f;
        }
        __syncthreads();
        if (tid == 0) g[1] = fr_sub(st->claim, g[0]);
        __syncthreads();
        Fr v = block_finalise_round(TS, st, g, 4, a.rounds_off + (uint32_t)(a.li + t) * 128,
                                    a.chal_v + a.li + t);
        // fold the six tables: thread = (table, j)
        Fr folded = fr_zero();
        const int tb = tid >> 5, fj = tid & 31;
        if (tb < 6 && fj < half) {
            const Fr lo = T6[tb][fj], hi = T6[tb][fj + half];
            folded = fr_add(lo, fr_mul_ni(v, fr_sub(hi, lo)));
        }
        __syncthreads();
        if (tb < 6 && fj < half) T6[tb][fj] = folded;
        __syncthreads();
        cur = half;
    }
    // finals: aux~(0, v, wbar), aux~(1, v, wbar), aux~(0, v, Q+R-1) = 1 - (1 - sign)(v)
    if (tid == 0) {
        fin[0] = T6[0][0];
        fin[1] = T6[1][0];
        fin[2] = fr_sub(one, sc[T_NS]);
        for (int k = 0; k < 3; ++k) st->scal[4 + k] = fin[k];
    }
    __syncthreads();
    block_absorb_frs(TS, 'f', fin, 3, (uint32_t*)(st->proof + a.finals_off));
    block_challenges(TS, st, a.chal_rho, 3);   // rho0..2: one vector draw
    if (tid < 3) rho[tid] = st->chal[a.chal_rho + tid];
    __syncthreads();
    if (tid == 0) {
        Fr mc = fr_add(fr_add(fr_mul_ni(rho[0], fin[0]), fr_mul_ni(rho[1], fin[1])), fr_mul_ni(rho[2], fin[2]));
        st->claim = mc;
        Fr plain = fr_from_mont_ni(mc);
        uint32_t* dst = (uint32_t*)(st->proof + a.merge_claim_off);
        for (int l = 0; l < 8; ++l) dst[l] = plain.v[l];
    }
    // beta~(wbar, .) over j, built in place from the last coordinate upwards (into E[0..J))
    if (tid == 0) E[0] = one;
    __syncthreads();
    {
        int size = 1;
        for (int k = a.lj - 1; k >= 0; --k) {
            Fr u = st->chal[a.chal_v + a.li + k];
            Fr e, hi;
            if (tid < size) {
                e = E[tid];
                hi = fr_mul_ni(e, u);
            }
            __syncthreads();
            if (tid < size) {
                E[tid + size] = hi;
                E[tid] = fr_sub(e, hi);
            }
            size <<= 1;
            __syncthreads();
        }
    }
    // E(0, j) = rho0 beta(wbar, j) + rho2 [j == Q+R-1],  E(1, j) = rho1 beta(wbar, j)
    Fr bw = fr_zero();
    if (tid < 64 && tid < J) bw = E[tid];
    __syncthreads();
    if (tid < 64) {
        Fr e0 = fr_mul_ni(rho[0], bw);
        if (tid == nbits - 1) e0 = fr_add(e0, rho[2]);
        E[tid] = tid < J ? e0 : fr_zero();
        E[64 + tid] = tid < J ? fr_mul_ni(rho[1], bw) : fr_zero();
    }
    __syncthreads();
    // merge sumcheck over (k, j): k first, then the variables of j.  Compact the tables to
    // 2J entries when J < 64 so that halves are contiguous.
    if (J < 64) {
        Fr m1 = fr_zero(), e1 = fr_zero();
        if (tid < J) {
            m1 = M[64 + tid];
            e1 = E[64 + tid];
        }
        __syncthreads();
        if (tid < J) {
            M[J + tid] = m1;
            E[J + tid] = e1;
        }
        __syncthreads();
    }
    cur = 2 * J;
    for (int t = 0; t < 1 + a.lj; ++t) {
        const int half = cur >> 1;
        // wave w < 3: point x = w; lane = index below half (half <= 64)
        Fr f = fr_zero();
        if (wave < 3 && lane < half) {
            const Fr mlo = M[lane], mhi = M[lane + half], elo = E[lane], ehi = E[lane + half];
            if (wave == 0) f = fr_mul_ni(mlo, elo);
            else if (wave == 1) f = fr_mul_ni(mhi, ehi);
            else f = fr_mul_ni(fr_add(mhi, fr_sub(mhi, mlo)), fr_add(ehi, fr_sub(ehi, elo)));
        }
        if (wave < 3) {
            f = wave_sum_fr(f);
            if (lane == 0) g[wave] = f;
        }
        __syncthreads();
        Fr v = block_finalise_round(TS, st, g, 3, a.merge_rounds_off + (uint32_t)t * 96, a.chal_rho + 3 + t);
        Fr fm = fr_zero();
        const int tb = tid >> 6;
        if (tb < 2 && lane < half) {
            const Fr lo = tb == 0 ? M[lane] : E[lane], hi = tb == 0 ? M[lane + half] : E[lane + half];
            fm = fr_add(lo, fr_mul_ni(v, fr_sub(hi, lo)));
        }
        __syncthreads();
        if (tb < 2 && lane < half) {
            if (tb == 0) M[lane] = fm;
            else E[lane] = fm;
        }
        __syncthreads();
        cur = half;
    }
    if (tid == 0) {
        fin[0] = M[0];
        fin[1] = E[0];
        st->scal[7] = fin[0];
        st->scal[8] = fin[1];
    }
    __syncthreads();
    block_absorb_frs(TS, 'f', fin, 2, (uint32_t*)(st->proof + a.merge_finals_off));
    block_ts_store(TS, st);
}

unsigned blocks_for(uint64_t n, unsigned cap) {
    uint64_t b = (n + ZK_BLOCK - 1) / ZK_BLOCK;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (unsigned)b;
}

int log2u(uint64_t x) {
    int l = 0;
    while (((uint64_t)1 << l) < x) ++l;
    return l;
}

const uint32_t SC_MAGIC = 0x43534B5Au;

}  // namespace

int zk_zkrelu(zkdl_ctx* ctx, const int64_t* z_dev, const int64_t* ga_dev, uint64_t D, int Q, int R,
              int given_points) {
    const int nbits = Q + R;
    const int li = log2u(D);
    int lj = 0;
    while ((1 << lj) < nbits) ++lj;
    const int J = 1 << lj;
    const int has_ga = ga_dev != nullptr;
    const int need = 6 * li + 3 * lj + 6;
    if (ctx->n_chal + need > ZK_MAX_CHAL) return ZKDL_EINVAL;
    const int c0 = ctx->n_chal;
    const int c_uz = c0, c_ua = c0 + li, c_uga = c0 + 2 * li, c_ugz = c0 + 3 * li, c_ubin = c0 + 4 * li;
    const int c_r = c0 + 5 * li + lj, c_v = c_r + 2, c_rho = c_v + li + lj;
    ctx->n_chal += need;

    // proof layout
    const uint32_t claims_off = (uint32_t)ctx->proof_len;
    ctx->proof_len += 4 * 32;
    uint32_t hdr[4] = {SC_MAGIC, 3, 3, (uint32_t)(li + lj)};
    zk_write_proof_words(ctx, hdr, 4);
    const uint32_t claim0_off = (uint32_t)ctx->proof_len;
    const uint32_t rounds_off = claim0_off + 32;
    const uint32_t finals_off = rounds_off + (uint32_t)(li + lj) * 128;
    ctx->proof_len = finals_off + 3 * 32;
    uint32_t mhdr[4] = {SC_MAGIC, 2, 2, (uint32_t)(1 + lj)};
    zk_write_proof_words(ctx, mhdr, 4);
    const uint32_t mclaim_off = (uint32_t)ctx->proof_len;
    const uint32_t mrounds_off = mclaim_off + 32;
    const uint32_t mfinals_off = mrounds_off + (uint32_t)(1 + lj) * 96;
    ctx->proof_len = mfinals_off + 2 * 32;
    if (ctx->proof_len > (size_t)ZK_PROOF_CAP) return ZKDL_ESMALL;

    DevState* st = ctx->dev;
    if (given_points) zk_launch_draw(ctx, c_ubin, li + lj);
    else zk_launch_draw(ctx, c0, 5 * li + lj);

    // memory: 10 D-sized tables, beta_J, aux columns (2 * nbits columns of 36 B entries; the rows
    // are written once four challenges are bound, D/16 of them; fewer challenges if D < 16)
    // column chunks of round t (m pairs): few rows are split over more threads (rounds 0 and 1 take the
    // 64-bit words whole); every (pair index, chunk) thread pays the beta_I fold and the reductions on
    // top of its columns, so only until the machine is full (the context's fill threshold)
    const uint64_t fill_threads = ctx->zk_fill_threads ? ctx->zk_fill_threads : 1;
    auto chunks_of = [&](int t, uint64_t m, int* jc_out, int* ksplit_out) -> unsigned {
        int jc = nbits;
        if (t >= 2)
            while ((uint64_t)((nbits + jc - 1) / jc) * m < fill_threads && jc > 1) jc = (jc + 1) / 2;
        unsigned chunks = (unsigned)((nbits + jc - 1) / jc);
        // one column per thread and still not full: give the two slices their own threads as well
        const int ks = (t >= 2 && has_ga && jc == 1 && (uint64_t)chunks * m < fill_threads) ? 1 : 0;
        if (ks) chunks *= 2;
        if (jc_out) *jc_out = jc;
        if (ksplit_out) *ksplit_out = ks;
        return chunks;
    };
    // the columns are written after four challenges, or after five when round 4 can run on the
    // integers (whole columns per thread, column sums at hand); fewer for D < 16
    const bool round4_on_ints = li >= 5 && chunks_of(4, D >> 5, nullptr, nullptr) == 1;
    const int mat_bound = round4_on_ints ? 5 : li >= 4 ? 4 : li >= 3 ? 3 : 2;
    const uint64_t rows = li >= 3 ? D >> mat_bound : 1;
    const uint64_t aux_elems = (uint64_t)(has_ga ? 2 : 1) * nbits * rows;
    const uint64_t alt_rows = D >= 2 ? D / 2 : 1;   // second buffer of the beta_I folds
    void* mem = zk_alloc(ctx, (uint64_t)LIN_TABLES * D * 36 + 64 * 32 + alt_rows * 36 + (li >= 2 ? aux_elems * 36 : 0));
    // the first two i-rounds read the integers and take the equality tables over i as products
    // of two factors (the integers must exist in round 1, and the line values must fit 58 bits);
    // otherwise the five tables are built whole
    const int split = li >= 2 && nbits <= 56;
    const int hb = li / 2, lb = li - hb;
    const uint64_t nh = (uint64_t)1 << hb, nl = (uint64_t)1 << lb;
    // split: packed H and L of the five points, then as lazy limbs H, two buffers for the folded H, L
    const uint64_t split_words = 5 * (nh + nl) * 8 + 5 * (nh + 2 * ((nh + 1) / 2) + nl) * 9;
    void* beta_mem = zk_alloc(ctx, split ? split_words * 4 : (uint64_t)5 * D * 32);
    // column sums handed from round to round (from round 1 on): two sets of three tables; a round
    // with c chunks of m pairs leaves c m entries, and chunks appear only below the fill threshold
    constexpr unsigned PS_MAX_CHUNKS = 16;   // measured: 4 and 256 are slower (config 3: 2.96 and 5.2 ms against 2.83)
    const uint64_t ps_cap = li >= 4 ? ((D >> 2) > 4 * fill_threads ? (D >> 2) : 4 * fill_threads) : 0;
    void* ps_mem = ps_cap ? zk_alloc(ctx, 6 * ps_cap * 36) : nullptr;
    if (!mem || !beta_mem || (ps_cap && !ps_mem)) {
        zk_free(ctx, mem);
        zk_free(ctx, beta_mem);
        zk_free(ctx, ps_mem);
        return ZKDL_ENOMEM;
    }
    F9Tab ps_tab[2][3];
    for (int q = 0; q < 6; ++q) {
        ps_tab[q / 3][q % 3].p = (uint32_t*)ps_mem + (uint64_t)q * 9 * ps_cap;
        ps_tab[q / 3][q % 3].ps = ps_cap;
    }
    int ps_prev_chunks = 0;   // != 0: the previous round left its column sums in ps_tab[(t - 1) & 1]
    uint32_t* base = (uint32_t*)mem;
    ZkTabs tabs;
    for (int k = 0; k < LIN_TABLES; ++k) {
        tabs.t[k].p = base;
        tabs.t[k].ps = D;
        base += 9 * D;
    }
    Fr* bJ = (Fr*)base;
    base += 8 * 64;
    F9Tab bI_alt;
    bI_alt.p = base;
    bI_alt.ps = alt_rows;
    base += 9 * alt_rows;
    uint32_t* aux = base;
    ZkBeta8 beta8;
    for (int k = 0; k < 5; ++k) beta8.t[k] = make_tab((uint32_t*)beta_mem + (uint64_t)k * 8 * D, D);
    SplitEq sp0 = {}, sp1 = {}, sp2 = {};   // as built (H scaled after the weights are drawn); H with the challenges
                                            // bound so far, in turns
    SplitConvArgs sca = {};
    sp0.lb = sp1.lb = sp2.lb = lb;
    if (split) {
        uint32_t* q = (uint32_t*)beta_mem;
        for (int k = 0; k < 5; ++k) {
            sca.src[k] = make_tab(q, nh);
            sca.n[k] = nh;
            q += 8 * nh;
        }
        for (int k = 0; k < 5; ++k) {
            sca.src[5 + k] = make_tab(q, nl);
            sca.n[5 + k] = nl;
            q += 8 * nl;
        }
        for (int k = 0; k < 5; ++k) {
            sp0.H[k].p = q;
            sp0.H[k].ps = nh;
            q += 9 * nh;
            sca.dst[k] = sp0.H[k];
        }
        for (int k = 0; k < 5; ++k) {
            sp1.H[k].p = q;
            sp1.H[k].ps = (nh + 1) / 2;
            q += 9 * ((nh + 1) / 2);
        }
        for (int k = 0; k < 5; ++k) {
            sp2.H[k].p = q;
            sp2.H[k].ps = (nh + 1) / 2;
            q += 9 * ((nh + 1) / 2);
        }
        for (int k = 0; k < 5; ++k) {
            sp0.L[k].p = q;
            sp0.L[k].ps = nl;
            q += 9 * nl;
            sp1.L[k] = sp0.L[k];
            sp2.L[k] = sp0.L[k];
            sca.dst[5 + k] = sp0.L[k];
        }
    }

    // beta_J as an array of structures: one plane of J elements read through FrTab, then copied
    void* bj_tmp = zk_alloc(ctx, 64 * 32);
    int rc = bj_tmp ? ZKDL_OK : ZKDL_ENOMEM;
    FrTab bj_soa = make_tab(bj_tmp, J);
    if (rc == ZKDL_OK) {
        BetaJob jobs[11];
        int nj = 0;
        const int cpt[5] = {c_uz, c_ua, c_uga, c_ugz, c_ubin};
        for (int k = 0; k < 5; ++k) {
            if ((k == 2 || k == 3) && !has_ga) continue;
            if (split) {
                jobs[nj++] = BetaJob{st->chal + cpt[k], hb, sca.src[k]};
                jobs[nj++] = BetaJob{st->chal + cpt[k] + hb, lb, sca.src[5 + k]};
            } else {
                jobs[nj++] = BetaJob{st->chal + cpt[k], li, beta8.t[k]};
            }
        }
        jobs[nj++] = BetaJob{st->chal + c_ubin + li, lj, bj_soa};
        rc = zk_build_beta_many(ctx, jobs, nj);
    }
    if (rc != ZKDL_OK) {
        zk_free(ctx, bj_tmp);
        zk_free(ctx, mem);
        zk_free(ctx, beta_mem);
        zk_free(ctx, ps_mem);
        return rc;
    }
    zk_launch_soa_to_aos(ctx, bj_soa, J, bJ);
    if (split) {
        if (!has_ga)   // tables that are not built are not converted either
            for (int k = 2; k <= 3; ++k) sca.n[k] = sca.n[5 + k] = 0;
        hipLaunchKernelGGL(k_zk_split_convert, dim3(blocks_for(nh > nl ? nh : nl, 64), 10), dim3(ZK_BLOCK), 0, ctx->stream, sca);
    }

    PrepArgs pa;
    pa.z = z_dev;
    pa.ga = ga_dev;
    pa.D = D;
    pa.nbits = nbits;
    pa.r_bits = R;
    pa.beta = beta8;
    pa.tabs = tabs;
    const int lin_from_ints = split;
    pa.write_vals = !lin_from_ints;
    pa.sp = sp0;
    pa.part = ctx->partials;
    pa.st = st;
    // the integer kernel pays eight products per thread when a run ends: at least eight rows per thread
    unsigned nb = lin_from_ints ? blocks_for((D + 7) / 8, ZK_MAX_PART_BLOCKS) : blocks_for(D, ZK_MAX_PART_BLOCKS);
    if (lin_from_ints) hipLaunchKernelGGL(k_zk_prepare_int, dim3(nb), dim3(ZK_BLOCK), 0, ctx->stream, pa);
    else hipLaunchKernelGGL(k_zk_prepare, dim3(nb), dim3(ZK_BLOCK), 0, ctx->stream, pa);
    ClaimsArgs ca;
    ca.part = ctx->partials;
    ca.nblk = (int)nb;
    ca.st = st;
    ca.claims_off = claims_off;
    ca.claim0_off = claim0_off;
    ca.chal_r = c_r;
    hipLaunchKernelGGL(k_zk_claims, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ca);
    if (split)
        hipLaunchKernelGGL(k_zk_split_scale, dim3(blocks_for(nh, 64), 4), dim3(ZK_BLOCK), 0, ctx->stream, sp0, nh,
                           (const Fr*)st->weights, has_ga);
    else
        hipLaunchKernelGGL(k_zk_scale, dim3(blocks_for(D, 65536)), dim3(ZK_BLOCK), 0, ctx->stream, beta8, tabs, D,
                           (const Fr*)st->weights, has_ga);

    // Rounds that take the equality tables from their two factors: 0 and 1, and further rounds
    // while their variable lies in H and the round is large (its linear part is bound by the
    // table traffic then); the last of them writes the folded tables for the rounds after it.
    int sp_rounds = split ? 2 : 0;
    if (split)
        while (sp_rounds < hb && sp_rounds < li && (D >> (sp_rounds + 1)) >= 2 * fill_threads) ++sp_rounds;

    BinArgs ba;
    ba.z = z_dev;
    ba.ga = ga_dev;
    ba.aux = aux;
    ba.ps = rows;
    ba.nbits = nbits;
    ba.has_ga = has_ga;
    ba.bI = tabs.t[T_BI];
    ba.bI_out = bI_alt;
    ba.vprev = nullptr;
    ba.ksplit = 0;
    ba.bJ = bJ;
    ba.rp = &st->weights[4];
    ba.jc = nbits;
    ba.chal = nullptr;
    ba.m = 0;
    ba.part = nullptr;
    ba.split = 0;
    ba.sH = sp0.H[4];
    ba.sL = sp0.L[4];
    ba.s_lb = lb;

    for (int t = 0; t < li; ++t) {
        const uint64_t m = D >> (t + 1);
        ZkRoundArgs ra;
        ra.lin.tabs = tabs;
        ra.lin.m = m;
        ra.lin.chal = t > 0 ? &st->chal[c_v + t - 1] : nullptr;
        ra.lin.part = ctx->partials;
        ra.lin.has_ga = has_ga;
        ra.lin.from_ints = lin_from_ints && t <= 1;
        ra.lin.z = z_dev;
        ra.lin.ga = ga_dev;
        ra.lin.nbits = nbits;
        ra.lin.r_bits = R;
        const SplitEq& sp_t = t == 0 ? sp0 : (t & 1) ? sp1 : sp2;
        ra.lin.sp = sp_t;
        ra.lin.split_eq = t < sp_rounds;
        ra.lin.write_eq = t + 1 == sp_rounds;
        ba.split = t < sp_rounds;
        ba.sH = sp_t.H[4];
        // few pairs: 16 per block, spread over (table, pair) and (point, equation, pair) threads
        ra.lin_small = !ra.lin.from_ints && !ra.lin.split_eq && m <= (uint64_t)LIN_SMALL_PAIRS * (ZK_MAX_PART_BLOCKS / 2);
        const unsigned n_eq = has_ga ? 4 : 2;
        ra.lin.eq_blocks = blocks_for(m, ZK_MAX_PART_BLOCKS / 2 / n_eq);
        const unsigned nb_lin = ra.lin.from_ints ? n_eq * ra.lin.eq_blocks
                                : ra.lin_small       ? (unsigned)((m + LIN_SMALL_PAIRS - 1) / LIN_SMALL_PAIRS)
                                                     : blocks_for(m, ZK_MAX_PART_BLOCKS / 2);
        ra.nb_lin = nb_lin;
        // beta_I: round 0 reads the table as built; round t >= 1 reads what round t-1 left (the
        // table as built for t = 1), binds v_{t-1} and leaves the folded pair in the other buffer
        ba.bI = (t == 0 || (t & 1)) ? tabs.t[T_BI] : bI_alt;
        ba.bI_out = (t & 1) ? bI_alt : tabs.t[T_BI];
        ba.vprev = t > 0 ? &st->chal[c_v + t - 1] : nullptr;
        ba.m = m;
        ba.part = ctx->partials + (uint64_t)nb_lin * 4;
        int jc = nbits, ksplit = 0;
        const unsigned chunks = chunks_of(t, m, &jc, &ksplit);
        ba.ksplit = ksplit;
        const unsigned bx = blocks_for(m, ZK_MAX_PART_BLOCKS / 2 / chunks);
        const unsigned nb_bin = bx * chunks;
        ba.jc = jc;
        ba.chal = t == 0 ? nullptr : t < mat_bound ? &st->chal[c_v] : t > mat_bound ? &st->chal[c_v + t - 1] : nullptr;
        // column sums: rounds 1 and 3 compute theirs in full, a round that uses the previous round's
        // leaves its own for the next, as long as the columns are cut into few chunks
        const bool ps_ok = mat_bound >= 4 && t >= 1 && chunks <= PS_MAX_CHUNKS && (uint64_t)chunks * m <= ps_cap;
        const bool ps_use = ps_ok && t >= 2 && ps_prev_chunks != 0;
        const bool ps_produce = ps_ok && (t == 1 || t == 3 || ps_use);
        for (int q = 0; q < 3; ++q) {
            ba.ps_in[q] = ps_tab[(t + 1) & 1][q];
            ba.ps_out[q] = ps_tab[t & 1][q];
        }
        ba.ps_in_chunks = ps_prev_chunks;
        ba.ps_write = ps_produce ? 1 : 0;
        ps_prev_chunks = ps_produce ? (int)chunks : 0;
        ra.bin = ba;
        ra.bin_gx = bx;
        // algorithmic bytes: the linear tables (9 of them with G_A, 5 without) and beta_I in 36-byte
        // entries, the integers or the columns of the binarity part
        const double n_lin = has_ga ? 9.0 : 5.0, ns = has_ga ? 2.0 : 1.0;
        double bytes = n_lin * (t == 0 ? 72.0 : 216.0) * (double)m + (t == 0 ? 72.0 : 216.0) * (double)m;
        if (t == 0) bytes += ns * 16.0 * (double)m;
        else if (t == 1) bytes += ns * 32.0 * (double)m;
        else if (t == 2) bytes += ns * 64.0 * (double)m;
        else if (t < mat_bound) bytes += ns * (t == 3 ? 128.0 : 256.0) * (double)m;
        else bytes += ns * nbits * (t > mat_bound ? 216.0 : 72.0) * (double)m;
        zk_prof_begin(ctx, ZKDL_PROF_ZK_BIN, bytes);
        if (t == 0) launch_zk_round<0>(ctx, ra, nb_bin);
        else if (t == 1) launch_zk_round<1>(ctx, ra, nb_bin);
        else if (t == 2) {
            if (ps_use) launch_zk_round<8>(ctx, ra, nb_bin);
            else launch_zk_round<2>(ctx, ra, nb_bin);
        } else if (t == 3 && t < mat_bound) {
            if (ps_use) launch_zk_round<9>(ctx, ra, nb_bin);
            else launch_zk_round<5>(ctx, ra, nb_bin);
        } else if (t < mat_bound) {
            launch_zk_round<10>(ctx, ra, nb_bin);   // round 4 on the integers: mat_bound = 5 implies ps_use
        }
        else if (t == mat_bound && ps_use) launch_zk_round<6>(ctx, ra, nb_bin);
        else if (t == mat_bound) launch_zk_round<3>(ctx, ra, nb_bin);
        else if (ps_use) launch_zk_round<7>(ctx, ra, nb_bin);
        else launch_zk_round<4>(ctx, ra, nb_bin);
        zk_prof_end(ctx);
        // g(1) is taken from the running claim: the binarity kernels leave it out
        zk_launch_finalise(ctx, (int)(nb_lin + nb_bin), 4, c_v + t, rounds_off + (uint32_t)t * 128, 0, 0, 1);
        if (t + 1 < sp_rounds && (nh >> (t + 1)) >= 1) {   // the next round reads the H factors with v_t bound
            const SplitEq& sp_n = ((t + 1) & 1) ? sp1 : sp2;
            hipLaunchKernelGGL(k_zk_split_fold, dim3(blocks_for(nh >> (t + 1), 64), 5), dim3(ZK_BLOCK), 0, ctx->stream,
                               sp_t, sp_n, nh >> (t + 1), (const Fr*)&st->chal[c_v + t], has_ga);
        }
        if (t + 1 == mat_bound) {
            // bind the first challenges: bits -> field elements, one look-up per entry
            int jc = nbits;
            while ((uint64_t)((nbits + jc - 1) / jc) * m < 262144 && jc > 1) jc = (jc + 1) / 2;
            unsigned chunks = (unsigned)((nbits + jc - 1) / jc);
            ba.jc = jc;
            ba.ksplit = 0;
            ba.chal = &st->chal[c_v];
            ba.m = m;
            if (mat_bound == 2)
                hipLaunchKernelGGL(k_zk_mat2, dim3(blocks_for(m, 16384), chunks), dim3(ZK_BLOCK), 0, ctx->stream, ba);
            else if (mat_bound == 5)
                hipLaunchKernelGGL(k_zk_mat5, dim3(blocks_for(m, 16384)), dim3(ZK_BLOCK), 0, ctx->stream, ba);
            else if (mat_bound == 4)
                hipLaunchKernelGGL(k_zk_mat4, dim3(blocks_for(m, 16384), chunks), dim3(ZK_BLOCK), 0, ctx->stream, ba);
            else
                hipLaunchKernelGGL(k_zk_mat3, dim3(blocks_for(m, 16384), chunks), dim3(ZK_BLOCK), 0, ctx->stream, ba);
        }
    }
    TailArgs ta;
    ta.tabs = tabs;
    if (li >= 2 && ((li - 1) & 1)) ta.tabs.t[T_BI] = bI_alt;   // where the last round left beta_I
    ta.bin = ba;
    ta.li = li;
    ta.lj = lj;
    ta.mat_bound = mat_bound;
    ta.q_bits = Q;
    ta.r_bits = R;
    ta.st = st;
    ta.chal_v = c_v;
    ta.chal_rho = c_rho;
    ta.rounds_off = rounds_off;
    ta.finals_off = finals_off;
    ta.merge_claim_off = mclaim_off;
    ta.merge_rounds_off = mrounds_off;
    ta.merge_finals_off = mfinals_off;
    hipLaunchKernelGGL(k_zk_tail, dim3(1), dim3(TAIL_THREADS), 0, ctx->stream, ta);
    zk_free(ctx, bj_tmp);
    zk_free(ctx, mem);
    zk_free(ctx, beta_mem);
    zk_free(ctx, ps_mem);
    return ZKDL_OK;
}
