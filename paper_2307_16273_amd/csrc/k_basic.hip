// Conversion into Fr, equality-polynomial tables, and MLE partial evaluation
// (Eq. multilinear-extension, Sec. 2.2) for gfx950.
#include "zkdl_internal.h"

// ---------------------------------------------------------------------------
// integer / byte sources -> Fr (Montgomery, SoA)
// ---------------------------------------------------------------------------
template <int KIND>
__device__ __forceinline__ Fr load_src(const void* src, uint64_t i) {
    if (KIND == TK_I32) return fr_from_i64((int64_t)((const int32_t*)src)[i]);
    if (KIND == TK_I64) return fr_from_i64(((const int64_t*)src)[i]);
    if (KIND == TK_FR) {
        // never reached: Fr sources are read through FrTab
        return fr_zero();
    }
    // raw 32-byte little-endian values
    const uint32_t* p = (const uint32_t*)src + 8 * i;
    Fr x;
#pragma unroll
    for (int l = 0; l < 8; ++l) x.v[l] = p[l];
    return fr_to_mont(x);
}

constexpr int KIND_LE = 3;

template <int KIND>
__global__ __launch_bounds__(ZK_BLOCK) void k_convert(const void* src, uint64_t n, FrTab out) {
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n;
         i += (uint64_t)gridDim.x * blockDim.x)
        tab_st(out, i, load_src<KIND>(src, i));
}

static unsigned grid_for(uint64_t n, unsigned cap = 65536) {
    uint64_t b = (n + ZK_BLOCK - 1) / ZK_BLOCK;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (unsigned)b;
}

// the column sums of the lazy partial-evaluation kernels stay in range for this many elements per thread
constexpr uint64_t PE_LAZY_MAX_CHUNK = 4096;

void zk_launch_convert(zkdl_ctx* ctx, const void* src, int kind, uint64_t n, FrTab out) {
    unsigned g = grid_for(n);
    if (kind == TK_I32)
        hipLaunchKernelGGL(k_convert<TK_I32>, dim3(g), dim3(ZK_BLOCK), 0, ctx->stream, src, n, out);
    else if (kind == TK_I64)
        hipLaunchKernelGGL(k_convert<TK_I64>, dim3(g), dim3(ZK_BLOCK), 0, ctx->stream, src, n, out);
    else
        hipLaunchKernelGGL(k_convert<KIND_LE>, dim3(g), dim3(ZK_BLOCK), 0, ctx->stream, src, n, out);
}

__global__ __launch_bounds__(ZK_BLOCK) void k_download(FrTab in, uint64_t n, uint32_t* out) {
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n;
         i += (uint64_t)gridDim.x * blockDim.x) {
        Fr x = fr_from_mont(tab_ld(in, i));
#pragma unroll
        for (int l = 0; l < 8; ++l) out[8 * i + l] = x.v[l];
    }
}

void zk_launch_download(zkdl_ctx* ctx, FrTab in, uint64_t n, uint8_t* out_le_dev) {
    hipLaunchKernelGGL(k_download, dim3(grid_for(n)), dim3(ZK_BLOCK), 0, ctx->stream, in, n,
                       (uint32_t*)out_le_dev);
}

__global__ void k_points_to_mont(const uint32_t* le, int n, Fr* out) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        Fr x;
#pragma unroll
        for (int l = 0; l < 8; ++l) x.v[l] = le[8 * i + l];
        out[i] = fr_to_mont(x);
    }
}

void zk_launch_points_to_mont(zkdl_ctx* ctx, const uint8_t* le_dev, int n, Fr* out) {
    if (n <= 0) return;
    hipLaunchKernelGGL(k_points_to_mont, dim3((n + 63) / 64), dim3(64), 0, ctx->stream,
                       (const uint32_t*)le_dev, n, out);
}

// chal[dst + i] (and its little-endian copy) = the i-th given coordinate: taken from canonical
// little-endian bytes, or, with le == nullptr, a copy of chal[idx.v[i]]
__global__ void k_chal_set(DevState* st, int dst, int n, const uint32_t* le, ChalIdx idx) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    Fr x, xm;
    if (le) {
#pragma unroll
        for (int l = 0; l < 8; ++l) x.v[l] = le[8 * i + l];
        xm = fr_to_mont(x);
    } else {
        xm = st->chal[idx.v[i]];
        x = fr_from_mont(xm);
    }
    st->chal[dst + i] = xm;
    uint32_t* out = (uint32_t*)(st->chal_le + 32 * (size_t)(dst + i));
#pragma unroll
    for (int l = 0; l < 8; ++l) out[l] = x.v[l];
}

void zk_launch_chal_set(zkdl_ctx* ctx, int dst, int n, const uint8_t* le_dev, const ChalIdx* idx) {
    if (n <= 0) return;
    ChalIdx none = {};
    hipLaunchKernelGGL(k_chal_set, dim3((n + 63) / 64), dim3(64), 0, ctx->stream, ctx->dev, dst, n,
                       (const uint32_t*)le_dev, idx ? *idx : none);
}

// ---------------------------------------------------------------------------
// beta~(u, .): the multilinear extension of the equality indicator (Sec. 2.2),
// beta~(u, b) = prod_k (u_k b_k + (1 - u_k)(1 - b_k)), u_0 <-> most significant bit.
// Built from the last coordinate upwards so that each step is in place:
//   T[b + size] = T[b] * u_k ;  T[b] = T[b] - T[b + size]
// ---------------------------------------------------------------------------
constexpr int BETA_SMALL_MAX = 11;   // one block builds up to 2^11 entries

__global__ __launch_bounds__(ZK_BLOCK) void k_beta_small(const Fr* point, int m, FrTab out) {
    if (threadIdx.x == 0) tab_st(out, 0, fr_one());
    __syncthreads();
    uint64_t size = 1;
    for (int k = m - 1; k >= 0; --k) {
        Fr u = point[k];
        for (uint64_t b = threadIdx.x; b < size; b += blockDim.x) {
            Fr e = tab_ld(out, b);
            Fr hi = fr_mul(e, u);
            tab_st(out, b + size, hi);
            tab_st(out, b, fr_sub(e, hi));
        }
        size <<= 1;
        __syncthreads();
    }
}

// out[(h << lo_bits) | l] = hi[h] * lo[l]
__global__ __launch_bounds__(ZK_BLOCK) void k_beta_outer(FrTab hi, FrTab lo, int lo_bits, uint64_t n,
                                                         FrTab out) {
    uint64_t mask = ((uint64_t)1 << lo_bits) - 1;
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n;
         i += (uint64_t)gridDim.x * blockDim.x) {
        Fr a = tab_ld(hi, i >> lo_bits);
        Fr b = tab_ld(lo, i & mask);
        tab_st(out, i, fr_mul(a, b));
    }
}

int zk_build_beta(zkdl_ctx* ctx, const Fr* point, int m, FrTab out) {
    if (m <= BETA_SMALL_MAX) {
        hipLaunchKernelGGL(k_beta_small, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, point, m, out);
        return ZKDL_OK;
    }
    int hb = m / 2, lb = m - hb;
    uint64_t hn = (uint64_t)1 << hb, ln = (uint64_t)1 << lb;
    void* tmp = zk_alloc(ctx, (hn + ln) * 32);
    if (!tmp) return ZKDL_ENOMEM;
    FrTab th = make_tab(tmp, hn);
    FrTab tl = make_tab((uint32_t*)tmp + 8 * hn, ln);
    int rc = zk_build_beta(ctx, point, hb, th);
    if (rc == ZKDL_OK) rc = zk_build_beta(ctx, point + hb, lb, tl);
    if (rc == ZKDL_OK) {
        uint64_t n = (uint64_t)1 << m;
        hipLaunchKernelGGL(k_beta_outer, dim3(grid_for(n)), dim3(ZK_BLOCK), 0, ctx->stream, th, tl,
                           lb, n, out);
    }
    zk_free(ctx, tmp);   // stream-ordered reuse: later kernels on the same stream run after this one
    return rc;
}

// ---- several tables at once: one launch for all doubling builds, one for all outer products ----
constexpr int BETA_MAX_SMALL = 16;
constexpr int BETA_MAX_OUTER = 8;

struct BetaSmallBatch {
    const Fr* point[BETA_MAX_SMALL];
    int m[BETA_MAX_SMALL];
    FrTab out[BETA_MAX_SMALL];
};

__global__ __launch_bounds__(ZK_BLOCK) void k_beta_small_batch(BetaSmallBatch bb) {
    const Fr* point = bb.point[blockIdx.x];
    const int m = bb.m[blockIdx.x];
    const FrTab out = bb.out[blockIdx.x];
    if (threadIdx.x == 0) tab_st(out, 0, fr_one());
    __syncthreads();
    uint64_t size = 1;
    for (int k = m - 1; k >= 0; --k) {
        Fr u = point[k];
        for (uint64_t b = threadIdx.x; b < size; b += blockDim.x) {
            Fr e = tab_ld(out, b);
            Fr hi = fr_mul(e, u);
            tab_st(out, b + size, hi);
            tab_st(out, b, fr_sub(e, hi));
        }
        size <<= 1;
        __syncthreads();
    }
}

struct BetaOuterBatch {
    FrTab hi[BETA_MAX_OUTER], lo[BETA_MAX_OUTER], out[BETA_MAX_OUTER];
    int lo_bits[BETA_MAX_OUTER];
    uint64_t n[BETA_MAX_OUTER];
};

__global__ __launch_bounds__(ZK_BLOCK) void k_beta_outer_batch(BetaOuterBatch ob) {
    const int q = blockIdx.y;
    const FrTab hi = ob.hi[q], lo = ob.lo[q], out = ob.out[q];
    const int lo_bits = ob.lo_bits[q];
    const uint64_t n = ob.n[q], mask = ((uint64_t)1 << lo_bits) - 1;
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n;
         i += (uint64_t)gridDim.x * blockDim.x)
        tab_st(out, i, fr_mul(tab_ld(hi, i >> lo_bits), tab_ld(lo, i & mask)));
}

int zk_build_beta_many(zkdl_ctx* ctx, const BetaJob* jobs, int n) {
    BetaSmallBatch sb;
    BetaOuterBatch ob;
    int ns = 0, no = 0;
    uint64_t tmp_elems = 0, max_n = 0;
    for (int i = 0; i < n; ++i) {
        const int m = jobs[i].m;
        if (m > BETA_SMALL_MAX && m <= 2 * BETA_SMALL_MAX) tmp_elems += ((uint64_t)1 << (m / 2)) + ((uint64_t)1 << (m - m / 2));
    }
    void* tmp = tmp_elems ? zk_alloc(ctx, tmp_elems * 32) : nullptr;
    if (tmp_elems && !tmp) return ZKDL_ENOMEM;
    uint32_t* tp = (uint32_t*)tmp;
    int rc = ZKDL_OK;
    for (int i = 0; i < n && rc == ZKDL_OK; ++i) {
        const int m = jobs[i].m;
        const bool split = m > BETA_SMALL_MAX && m <= 2 * BETA_SMALL_MAX;
        if (m > 2 * BETA_SMALL_MAX || ns + (split ? 2 : 1) > BETA_MAX_SMALL || (split && no + 1 > BETA_MAX_OUTER)) {
            rc = zk_build_beta(ctx, jobs[i].point, m, jobs[i].out);   // large or surplus tables: one by one
            continue;
        }
        if (!split) {
            sb.point[ns] = jobs[i].point;
            sb.m[ns] = m;
            sb.out[ns] = jobs[i].out;
            ++ns;
            continue;
        }
        const int hb = m / 2, lb = m - hb;
        const uint64_t hn = (uint64_t)1 << hb, ln = (uint64_t)1 << lb;
        const FrTab th = make_tab(tp, hn);
        tp += 8 * hn;
        const FrTab tl = make_tab(tp, ln);
        tp += 8 * ln;
        sb.point[ns] = jobs[i].point;
        sb.m[ns] = hb;
        sb.out[ns] = th;
        ++ns;
        sb.point[ns] = jobs[i].point + hb;
        sb.m[ns] = lb;
        sb.out[ns] = tl;
        ++ns;
        ob.hi[no] = th;
        ob.lo[no] = tl;
        ob.out[no] = jobs[i].out;
        ob.lo_bits[no] = lb;
        ob.n[no] = (uint64_t)1 << m;
        if (ob.n[no] > max_n) max_n = ob.n[no];
        ++no;
    }
    if (rc == ZKDL_OK && ns > 0)
        hipLaunchKernelGGL(k_beta_small_batch, dim3(ns), dim3(ZK_BLOCK), 0, ctx->stream, sb);
    if (rc == ZKDL_OK && no > 0)
        hipLaunchKernelGGL(k_beta_outer_batch, dim3(grid_for(max_n, 4096), no), dim3(ZK_BLOCK), 0, ctx->stream, ob);
    zk_free(ctx, tmp);   // stream-ordered reuse
    return rc;
}

// ---------------------------------------------------------------------------
// partial evaluation: out[o, i] = sum_a beta[a] * T[o, a, i]
// ---------------------------------------------------------------------------
template <int KIND>
__device__ __forceinline__ Fr pe_load(const void* src, uint64_t idx) {
    if (KIND == TK_FR) {
        const FrTab* t = (const FrTab*)src;
        return tab_ld(*t, idx);
    }
    return load_src<KIND>(src, idx);
}

struct PeArgs {
    const void* src;   // integers, or unused for Fr
    FrTab fr_src;      // Fr source
    FrTab beta;
    FrTab out;         // chunk c of output element e at index c * (O*I) + e
    uint64_t O, A, I;
    uint64_t a_chunk;  // contracted-axis entries per chunk
};

template <int KIND>
__device__ __forceinline__ Fr pe_elem(const PeArgs& p, uint64_t idx) {
    if (KIND == TK_FR) return tab_ld(p.fr_src, idx);
    return load_src<KIND>(p.src, idx);
}

// one thread per output element (o, i): coalesced when I is large
template <int KIND>
__global__ __launch_bounds__(ZK_BLOCK) void k_pe_mid(PeArgs p) {
    uint64_t n_out = p.O * p.I;
    uint64_t a0 = (uint64_t)blockIdx.y * p.a_chunk;
    uint64_t a1 = a0 + p.a_chunk;
    if (a1 > p.A) a1 = p.A;
    for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < n_out;
         e += (uint64_t)gridDim.x * blockDim.x) {
        uint64_t o = e / p.I, i = e - o * p.I;
        Fr acc = fr_zero();
        for (uint64_t a = a0; a < a1; ++a) {
            Fr x = pe_elem<KIND>(p, (o * p.A + a) * p.I + i);
            acc = fr_add(acc, fr_mul(tab_ld(p.beta, a), x));
        }
        tab_st(p.out, (uint64_t)blockIdx.y * n_out + e, acc);
    }
}

__device__ __forceinline__ Fr wave_sum(Fr x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        Fr y;
#pragma unroll
        for (int l = 0; l < 8; ++l) y.v[l] = __shfl_down(x.v[l], off, 64);
        x = fr_add(x, y);
    }
    return x;   // lane 0 holds the sum
}

// innermost axis contracted (I == 1): one wave per (output row, chunk), lanes stride over a
template <int KIND>
__global__ __launch_bounds__(ZK_BLOCK) void k_pe_inner(PeArgs p) {
    const int lane = threadIdx.x & 63;
    uint64_t wave = (blockIdx.x * (uint64_t)blockDim.x + threadIdx.x) >> 6;
    uint64_t n_waves = ((uint64_t)gridDim.x * blockDim.x) >> 6;
    uint64_t chunks = (p.A + p.a_chunk - 1) / p.a_chunk;
    uint64_t n_items = p.O * chunks;
    for (uint64_t it = wave; it < n_items; it += n_waves) {
        uint64_t c = it / p.O, o = it - c * p.O;
        uint64_t a0 = c * p.a_chunk, a1 = a0 + p.a_chunk;
        if (a1 > p.A) a1 = p.A;
        Fr acc = fr_zero();
        for (uint64_t a = a0 + lane; a < a1; a += 64) {
            Fr x = pe_elem<KIND>(p, o * p.A + a);
            acc = fr_add(acc, fr_mul(tab_ld(p.beta, a), x));
        }
        acc = wave_sum(acc);
        if (lane == 0) tab_st(p.out, c * p.O + o, acc);
    }
}

// Lazy variants: the products of one output are summed as 64-bit columns of 29-bit limb
// products and reduced once (f9_cols_*, f9_redc), instead of one Montgomery product and one
// modular addition per source element.  Thread per output element (o, i), block = 256 consecutive
// outputs; blockIdx.y selects the chunk of the contracted axis; beta_a is the same for every thread
// of an iteration and is unpacked once per block into LDS.
//
// Fr source: sum_a beta_a T_a, 81 multiply-adds per element, both in Montgomery form, so the
// reduced sum is the Montgomery form of the result.
// (int32 sources: k_pe_mid_i32 and k_pe_inner_i32_lazy below; there x_a is a plain integer, nine
// multiply-adds per element, and the sum is "beta times integer" already.)
constexpr int PE_FR_TILE = 256;   // entries of beta unpacked into LDS at a time
template <int KIND>
__global__ __launch_bounds__(ZK_BLOCK) void k_pe_mid_lazy(PeArgs p) {
    static_assert(KIND == TK_FR, "Fr sources only");
    __shared__ uint32_t sb[9][PE_FR_TILE];
    const uint64_t n_out = p.O * p.I;
    const uint64_t a0 = (uint64_t)blockIdx.y * p.a_chunk;
    uint64_t a1 = a0 + p.a_chunk;
    if (a1 > p.A) a1 = p.A;
    const uint64_t nblk = (n_out + ZK_BLOCK - 1) / ZK_BLOCK;
    for (uint64_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
        const uint64_t e = blk * ZK_BLOCK + threadIdx.x;
        const bool live = e < n_out;
        const uint64_t o = live ? e / p.I : 0, i = live ? e - o * p.I : 0;
        uint64_t c[17];
#pragma unroll
        for (int k = 0; k < 17; ++k) c[k] = 0;
        int pending = 0;
        for (uint64_t at = a0; at < a1; at += PE_FR_TILE) {
            const int na = (int)(a1 - at < PE_FR_TILE ? a1 - at : PE_FR_TILE);
            __syncthreads();   // the previous tile is no longer read
            if ((int)threadIdx.x < na) {   // beta of the tile, unpacked once per block (every thread reads the same entry)
                const F9 b9 = fr_unpack(tab_ld(p.beta, at + threadIdx.x));
#pragma unroll
                for (int l = 0; l < 9; ++l) sb[l][threadIdx.x] = b9.v[l];
            }
            __syncthreads();
            if (live) {
#pragma unroll 2
                for (int k = 0; k < na; ++k) {
                    F9 b9;
#pragma unroll
                    for (int l = 0; l < 9; ++l) b9.v[l] = sb[l][k];
                    const F9 x9 = fr_unpack(tab_ld(p.fr_src, (o * p.A + at + k) * p.I + i));
                    f9_cols_mac(c, b9, x9);
                    if (++pending == 4) {
                        pending = 0;
                        f9_cols_norm<17>(c);
                    }
                }
            }
        }
        if (live) {
            f9_cols_norm<17>(c);
            tab_st(p.out, (uint64_t)blockIdx.y * n_out + e, f9_to_fr(f9_norm_reduce(f9_redc(c))));
        }
    }
}

// Middle axis contracted, int32 source: thread = output (o, i), block = 256 consecutive outputs.
// beta of the chunk is unpacked once per block into LDS (every thread reads the same entry of an
// iteration); the integers of eight rows are requested together before they are used; the
// products beta_a x_a (29-bit limb by signed 32-bit integer) are added into ten signed 64-bit
// columns, carried every fourth element.  The sum is "beta times integer", a Montgomery form
// already: an offset 2^56 2^261 makes it non-negative, it is reduced (divide by 2^261),
// multiplied back by 2^522 mod r, and the offset's residue is taken off again.
constexpr int PE_MID_TILE = 256;
__global__ __launch_bounds__(ZK_BLOCK) void k_pe_mid_i32(PeArgs p) {
    __shared__ uint32_t sb[9][PE_MID_TILE];
    const uint64_t n_out = p.O * p.I;
    const uint64_t a0 = (uint64_t)blockIdx.y * p.a_chunk;
    uint64_t a1 = a0 + p.a_chunk;
    if (a1 > p.A) a1 = p.A;
    const int32_t* src = (const int32_t*)p.src;
    const uint64_t nblk = (n_out + ZK_BLOCK - 1) / ZK_BLOCK;
    for (uint64_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
        const uint64_t e = blk * ZK_BLOCK + threadIdx.x;
        const bool live = e < n_out;
        const uint64_t o = live ? e / p.I : 0, i = live ? e - o * p.I : 0;
        const int32_t* col = src + (o * p.A) * p.I + i;
        int64_t c[10];
#pragma unroll
        for (int k = 0; k < 10; ++k) c[k] = 0;
        for (uint64_t at = a0; at < a1; at += PE_MID_TILE) {
            const int na = (int)(a1 - at < PE_MID_TILE ? a1 - at : PE_MID_TILE);
            __syncthreads();   // the previous tile is no longer read
            if ((int)threadIdx.x < na) {
                const F9 b9 = fr_unpack(tab_ld(p.beta, at + threadIdx.x));
#pragma unroll
                for (int l = 0; l < 9; ++l) sb[l][threadIdx.x] = b9.v[l];
            }
            __syncthreads();
            if (live) {
                for (int k0 = 0; k0 < na; k0 += 8) {
                    int32_t x[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) x[u] = k0 + u < na ? col[(at + k0 + u) * p.I] : 0;
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int k = k0 + u < na ? k0 + u : 0;
#pragma unroll
                        for (int l = 0; l < 9; ++l) c[l] += (int64_t)(int32_t)sb[l][k] * (int64_t)x[u];
                        if ((u & 3) == 3) {   // four products below 2^60 in magnitude per column
#pragma unroll
                            for (int l = 0; l + 1 < 10; ++l) {
                                c[l + 1] += c[l] >> 29;
                                c[l] &= (int64_t)frc::M29;
                            }
                        }
                    }
                }
            }
        }
        if (live) {
            // |sum| < 2^286 (chunk length), chunks of at most 2^27 entries: with the offset the top column is positive
            uint64_t cols[17];
#pragma unroll
            for (int k = 0; k < 17; ++k) cols[k] = k < 10 ? (uint64_t)c[k] : 0;
            cols[9] += (uint64_t)1 << 56;
            const F9 r2 = fr_unpack(fr_const(frc::R2));
            F9 off = f9_zero();
            off.v[1] = 1u << 27;                                  // 2^56 as plain limbs
            const F9 koff = f9_mul(off, r2);                      // 2^56 2^261 mod r (up to a multiple of r), below 2r
            const F9 val = f9_mul(f9_redc(cols), r2);             // normal, below 2r
            tab_st(p.out, (uint64_t)blockIdx.y * n_out + e, f9_to_fr(f9_sub(val, koff)));
        }
    }
}

// Innermost axis contracted, int32 source: one wave per tile of 64 output rows and one chunk
// of the axis.  The tile of integers is read row by row (each row segment is contiguous, so
// the loads coalesce; all 64 rows are requested before the first is used) and transposed through LDS; then
// lane = row, and beta_a is the same for all lanes of an iteration.  Same arithmetic as
// k_pe_mid_i32: ten signed 64-bit columns, nine multiply-adds per element, carried every fourth
// element, the offset 2^56 2^261 at the end.
constexpr int PE_INNER_ROWS = 64;   // rows of a tile requested together: the whole tile (16 KB in flight per wave)
__global__ __launch_bounds__(64) void k_pe_inner_i32_lazy(PeArgs p) {
    __shared__ int32_t tile[64][65];
    __shared__ F9 sb[64];
    const int lane = threadIdx.x;
    const uint64_t row0 = (uint64_t)blockIdx.x * 64;
    const uint64_t a0 = (uint64_t)blockIdx.y * p.a_chunk;
    uint64_t a1 = a0 + p.a_chunk;
    if (a1 > p.A) a1 = p.A;
    const int32_t* src = (const int32_t*)p.src;
    int64_t c[10];
#pragma unroll
    for (int k = 0; k < 10; ++k) c[k] = 0;
    const int rows_here = (int)(p.O - row0 < 64 ? p.O - row0 : 64);
    for (uint64_t at = a0; at < a1; at += 64) {
        const int na = (int)(a1 - at < 64 ? a1 - at : 64);
        if (lane < na) sb[lane] = fr_unpack(tab_ld(p.beta, at + lane));
        const int32_t* seg = src + row0 * p.A + at + lane;
        for (int r0 = 0; r0 < rows_here; r0 += PE_INNER_ROWS) {
            int32_t x[PE_INNER_ROWS];
#pragma unroll
            for (int u = 0; u < PE_INNER_ROWS; ++u)
                x[u] = (lane < na && r0 + u < rows_here) ? seg[(uint64_t)(r0 + u) * p.A] : 0;
#pragma unroll
            for (int u = 0; u < PE_INNER_ROWS; ++u) tile[r0 + u][lane] = x[u];
        }
        __syncthreads();
        if (lane < rows_here) {
            for (int k0 = 0; k0 < na; k0 += 4) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int k = k0 + u < na ? k0 + u : 0;
                    const int64_t x = k0 + u < na ? (int64_t)tile[lane][k] : 0;
                    const F9 b9 = sb[k];
#pragma unroll
                    for (int l = 0; l < 9; ++l) c[l] += (int64_t)(int32_t)b9.v[l] * x;
                }
                // four products below 2^60 in magnitude per column
#pragma unroll
                for (int l = 0; l + 1 < 10; ++l) {
                    c[l + 1] += c[l] >> 29;
                    c[l] &= (int64_t)frc::M29;
                }
            }
        }
        __syncthreads();
    }
    if (lane < rows_here) {
        // |sum| < 2^286 (chunks of at most 2^27 entries): with the offset the top column is positive
        uint64_t cols[17];
#pragma unroll
        for (int k = 0; k < 17; ++k) cols[k] = k < 10 ? (uint64_t)c[k] : 0;
        cols[9] += (uint64_t)1 << 56;
        const F9 r2 = fr_unpack(fr_const(frc::R2));
        F9 off = f9_zero();
        off.v[1] = 1u << 27;                                  // 2^56 as plain limbs
        const F9 koff = f9_mul(off, r2);                      // 2^56 2^261 mod r (up to a multiple of r), below 2r
        const F9 val = f9_mul(f9_redc(cols), r2);             // normal, below 2r
        tab_st(p.out, (uint64_t)blockIdx.y * p.O + row0 + lane, f9_to_fr(f9_sub(val, koff)));
    }
}

// out[e] = sum_c part[c * n + e]
__global__ __launch_bounds__(ZK_BLOCK) void k_sum_chunks(FrTab part, uint64_t n, uint64_t chunks,
                                                         FrTab out) {
    for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < n;
         e += (uint64_t)gridDim.x * blockDim.x) {
        Fr acc = tab_ld(part, e);
        for (uint64_t c = 1; c < chunks; ++c) acc = fr_add(acc, tab_ld(part, c * n + e));
        tab_st(out, e, acc);
    }
}

template <int KIND>
static void launch_pe(zkdl_ctx* ctx, bool inner, const PeArgs& p, dim3 grid) {
    if (inner)
        hipLaunchKernelGGL(k_pe_inner<KIND>, grid, dim3(ZK_BLOCK), 0, ctx->stream, p);
    else if (KIND == TK_I32)
        hipLaunchKernelGGL(k_pe_mid_i32, grid, dim3(ZK_BLOCK), 0, ctx->stream, p);
    else if (KIND == TK_FR && p.a_chunk <= PE_LAZY_MAX_CHUNK)
        hipLaunchKernelGGL(k_pe_mid_lazy<TK_FR>, grid, dim3(ZK_BLOCK), 0, ctx->stream, p);
    else
        hipLaunchKernelGGL(k_pe_mid<KIND>, grid, dim3(ZK_BLOCK), 0, ctx->stream, p);
}

int zk_partial_eval(zkdl_ctx* ctx, int kind, const void* src, uint64_t O, uint64_t A, uint64_t I,
                    FrTab beta, FrTab out) {
    PeArgs p;
    p.src = src;
    if (kind == TK_FR) p.fr_src = *(const FrTab*)src;
    else p.fr_src = make_tab(nullptr, 0);
    p.beta = beta;
    p.O = O;
    p.A = A;
    p.I = I;
    uint64_t n_out = O * I;
    const bool inner = (I == 1);
    if (inner && kind == TK_I32 && A >= 64) {
        // row tiles of 64 outputs x chunks of the axis, about a thousand single-wave blocks
        const uint64_t tiles = (O + 63) / 64;
        uint64_t chunks = 1;
        while (tiles * chunks < 1024 && A / (chunks * 2) >= 64) chunks *= 2;
        while (A / chunks > PE_LAZY_MAX_CHUNK) chunks *= 2;
        if (tiles <= 0x7fffffffu && chunks <= 65535) {
            p.a_chunk = (A + chunks - 1) / chunks;
            void* tmp = nullptr;
            if (chunks > 1) {
                tmp = zk_alloc(ctx, chunks * n_out * 32);
                if (!tmp) return ZKDL_ENOMEM;
                p.out = make_tab(tmp, chunks * n_out);
            } else {
                p.out = out;
            }
            zk_prof_begin(ctx, ZKDL_PROF_PARTIAL_EVAL, 4.0 * (double)O * (double)A + 32.0 * (double)A + 32.0 * (double)n_out);
            hipLaunchKernelGGL(k_pe_inner_i32_lazy, dim3((unsigned)tiles, (unsigned)chunks), dim3(64), 0, ctx->stream, p);
            zk_prof_end(ctx);
            if (chunks > 1) {
                hipLaunchKernelGGL(k_sum_chunks, dim3(grid_for(n_out)), dim3(ZK_BLOCK), 0, ctx->stream, p.out,
                                   n_out, chunks, out);
                zk_free(ctx, tmp);
            }
            return ZKDL_OK;
        }
    }
    // split the contracted axis until there is enough parallel work: the thread-per-output
    // kernels hide their load latency only with several waves per SIMD (~256k threads)
    uint64_t units = inner ? n_out * 64 : n_out;
    uint64_t chunks = 1;
    const uint64_t want_units = inner ? 65536 : 262144;
    while (units * chunks < want_units && chunks * 2 <= A && (A / (chunks * 2)) >= (inner ? 64u : 4u)) chunks *= 2;
    while (!inner && A / chunks > PE_LAZY_MAX_CHUNK && chunks < 32768) chunks *= 2;
    p.a_chunk = (A + chunks - 1) / chunks;
    void* tmp = nullptr;
    if (chunks > 1) {
        tmp = zk_alloc(ctx, chunks * n_out * 32);
        if (!tmp) return ZKDL_ENOMEM;
        p.out = make_tab(tmp, chunks * n_out);
    } else {
        p.out = out;
    }
    dim3 grid;
    if (inner) {
        uint64_t waves = n_out * chunks;
        grid = dim3(grid_for(waves * 64, 16384));
    } else {
        grid = dim3(grid_for(n_out, 16384), (unsigned)chunks);
    }
    // algorithmic bytes: the source once, beta once per (outer, inner) tile is cached: count it once, the output
    const double esz = kind == TK_FR ? 32.0 : kind == TK_I32 ? 4.0 : 8.0;
    zk_prof_begin(ctx, ZKDL_PROF_PARTIAL_EVAL, esz * (double)O * (double)A * (double)I + 32.0 * (double)A + 32.0 * (double)n_out);
    if (kind == TK_FR) launch_pe<TK_FR>(ctx, inner, p, grid);
    else if (kind == TK_I32) launch_pe<TK_I32>(ctx, inner, p, grid);
    else launch_pe<TK_I64>(ctx, inner, p, grid);
    zk_prof_end(ctx);
    if (chunks > 1) {
        hipLaunchKernelGGL(k_sum_chunks, dim3(grid_for(n_out)), dim3(ZK_BLOCK), 0, ctx->stream, p.out,
                           n_out, chunks, out);
        zk_free(ctx, tmp);
    }
    return ZKDL_OK;
}

// out[r * inner + i] = src[r] : the stack-axis table beta~(w, n) seen over (n, i)
__global__ __launch_bounds__(ZK_BLOCK) void k_broadcast_rows(FrTab src, uint64_t rows, uint64_t inner,
                                                             FrTab out) {
    uint64_t n = rows * inner;
    for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < n;
         e += (uint64_t)gridDim.x * blockDim.x)
        tab_st(out, e, tab_ld(src, e / inner));
}

void zk_launch_broadcast_rows(zkdl_ctx* ctx, FrTab src, uint64_t rows, uint64_t inner, FrTab out) {
    hipLaunchKernelGGL(k_broadcast_rows, dim3(grid_for(rows * inner)), dim3(ZK_BLOCK), 0, ctx->stream,
                       src, rows, inner, out);
}

// out[r] = src[r + 1] unless r is the last slot of its period, where out[r] = 0:
// the stack re-indexing "layer l <- layer l+1" of the gradA family
__global__ __launch_bounds__(ZK_BLOCK) void k_shift_rows(FrTab src, uint64_t rows, uint64_t inner,
                                                         uint32_t period, FrTab out) {
    uint64_t n = rows * inner;
    for (uint64_t e = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; e < n;
         e += (uint64_t)gridDim.x * blockDim.x) {
        uint64_t r = e / inner;
        bool last = (r % period) == period - 1;
        tab_st(out, e, last ? fr_zero() : tab_ld(src, e + inner));
    }
}

void zk_launch_shift_rows(zkdl_ctx* ctx, FrTab src, uint64_t rows, uint64_t inner, uint32_t period,
                          FrTab out) {
    hipLaunchKernelGGL(k_shift_rows, dim3(grid_for(rows * inner)), dim3(ZK_BLOCK), 0, ctx->stream, src,
                       rows, inner, period, out);
}

// small SoA table -> array of structures (tables that single-block kernels index directly)
__global__ void k_soa_to_aos(FrTab in, int n, Fr* out) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = tab_ld(in, i);
}

void zk_launch_soa_to_aos(zkdl_ctx* ctx, FrTab in, int n, Fr* out) {
    hipLaunchKernelGGL(k_soa_to_aos, dim3((n + 63) / 64), dim3(64), 0, ctx->stream, in, n, out);
}
