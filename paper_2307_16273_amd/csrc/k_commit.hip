// Pedersen commitments on G1 of BLS12-381 and the row-wise commitment of a tensor (Sec. 2.3; Sec. 1.1;
// Protocol zkdl, the commit and proof-of-evaluation lines).
//
//   Commit(S; rho) = rho H + sum_i S_i G_i                                   (Sec. 2.3, additive notation)
//
// A tensor of 2^m quantised integers is laid out as R = 2^ceil(m/2) rows of C = 2^floor(m/2) columns and
// every row is committed with the same C generators and its own blinding scalar: the commitment has
// R = O(sqrt(size)) group elements (Sec. 1.1).  Generators are derived from a label by hashing to the
// curve (try-and-increment on SHA-256, cofactor cleared), so nobody knows a relation between them.
//
// Scalars are small: tensors are 32-bit (activations, weights, gradients) or 64-bit (pre-activations)
// signed integers, a negative entry x being the field element r - |x|, i.e. -|x| G.  The sum therefore
// runs over fixed-base window tables: for every generator the multiples d 2^(wk) G, d = 1..2^w - 1, k < bits/w,
// are built once with the key, in affine form (96 bytes an entry), and a commitment is a plain sum of one table
// entry per non-zero w-bit digit of |x| - no doublings and no buckets.  w = 12 while the tables stay below 16 GiB
// (1.2 MB per generator for 32-bit entries, 2.4 GB for 2048 columns: memory is what this GPU has), else w = 8.
// The blinding term rho H (rho a full field element) uses the same kind of table with 32 windows.  All sums use the complete projective formulas of fq.cuh: a row's sum may be
// taken in any order.
#include <string.h>
#include <new>
#include <vector>

#include "zkdl_internal.h"
#include "fq.cuh"

namespace {

constexpr int CK_WBITS = 8;                      // bits per window of the blinding scalar's table
constexpr int CK_DIGITS = (1 << CK_WBITS) - 1;   // its entries per window: d = 1..255
constexpr int CK_H_WINDOWS = 256 / CK_WBITS;     // windows of a 255-bit blinding scalar
constexpr int CK_WIDE_WBITS = 12;                // bits per window of a tensor entry when the tables fit CK_WIDE_MAX_BYTES
constexpr uint64_t CK_WIDE_MAX_BYTES = (uint64_t)16 << 30;   // up to 8192 columns of 32-bit entries (9.7 GB)
constexpr int CK_MAX_LABEL = 16;

struct LabelArg {
    uint8_t bytes[15 + CK_MAX_LABEL];   // "zkdl-mi355x/g1/" followed by the label
    uint32_t len;
};

// 2^384 * 2^812 mod q: brings the top 128 bits of a 512-bit hash into Montgomery form
// (fq_mul(hi, R2X) = hi 2^384 R mod q); checked against repeated doubling in zk_commit_selfcheck
__device__ __host__ inline Fq r2x_const() {
    Fq c = fq_const(fqc::R2);
    for (int i = 0; i < 384; ++i) c = fq_add(c, c);
    return c;
}

__device__ inline void sha_one_block(const uint8_t* msg, uint32_t len, uint32_t out[8]) {   // len <= 55
    uint32_t w[16];
    for (int i = 0; i < 16; ++i) w[i] = 0;
    for (uint32_t i = 0; i < len; ++i) w[i >> 2] |= (uint32_t)msg[i] << (24 - 8 * (i & 3));
    w[len >> 2] |= 0x80u << (24 - 8 * (len & 3));
    w[15] = len * 8;
    uint32_t h[8] = {0x6a09e667u, 0xbb67ae85u, 0x3c6ef372u, 0xa54ff53au, 0x510e527fu, 0x9b05688cu, 0x1f83d9abu, 0x5be0cd19u};
    sha::compress(h, w);
    for (int i = 0; i < 8; ++i) out[i] = h[i];
}

// plain a < plain b ?  (both below q, plain limbs)
__device__ inline bool limbs_less(const Fq& a, const Fq& b) {
    for (int i = fqc::L - 1; i >= 0; --i) {
        if (a.v[i] != b.v[i]) return a.v[i] < b.v[i];
    }
    return false;
}

// Generator `index` of the label: for ctr = 0, 1, .. the candidate x = int_be(SHA256(tag || u32be(index) ||
// u32be(ctr) || 0) || SHA256(.. || 1)) mod q; the first x for which x^3 + 4 is a square gives (x, y) with the
// smaller root y; cleared of the cofactor; a candidate that becomes the identity is skipped.
__global__ __launch_bounds__(64) void k_ck_generators(LabelArg label, uint64_t ncols, G1* gens, Fq r2x) {
    const uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (i > ncols) return;
    const uint32_t index = i < ncols ? (uint32_t)i : 0xFFFFFFFFu;   // the last one is the blinding generator H
    uint8_t msg[56];
    for (uint32_t b = 0; b < label.len; ++b) msg[b] = label.bytes[b];
    uint32_t at = label.len;
    for (int b = 0; b < 4; ++b) msg[at + b] = (uint8_t)(index >> (24 - 8 * b));
    at += 8;
    Fq four = fq_add(fq_one(), fq_one());
    four = fq_add(four, four);
    for (uint32_t ctr = 0;; ++ctr) {
        for (int b = 0; b < 4; ++b) msg[at - 4 + b] = (uint8_t)(ctr >> (24 - 8 * b));
        uint32_t dg[16];
        msg[at] = 0;
        sha_one_block(msg, at + 1, dg);
        msg[at] = 1;
        sha_one_block(msg, at + 1, dg + 8);
        // the 64 digest bytes as a big-endian integer: little-endian byte k is byte 63 - k of the digests
        uint8_t le[64];
        for (int k = 0; k < 64; ++k) {
            const int pos = 63 - k;
            le[k] = (uint8_t)(dg[pos >> 2] >> (24 - 8 * (pos & 3)));
        }
        uint8_t hi48[48];
        for (int k = 0; k < 48; ++k) hi48[k] = k < 16 ? le[48 + k] : 0;
        const Fq x = fq_add(fq_reduce_to_mont(fq_limbs_from_bytes(le)), fq_mul(fq_limbs_from_bytes(hi48), r2x));
        const Fq rhs = fq_add(fq_mul(fq_sqr(x), x), four);
        Fq y = fq_pow(rhs, fqc::EXP_SQRT);
        if (!fq_eq(fq_sqr(y), rhs)) continue;
        const Fq yn = fq_neg(y);
        if (limbs_less(fq_from_mont(yn), fq_from_mont(y))) y = yn;
        G1 p;
        p.X = x;
        p.Y = y;
        p.Z = fq_one();
        p = g1_mul_words(p, fqc::COFACTOR);
        if (fq_is_zero(p.Z)) continue;
        gens[i] = p;
        return;
    }
}

// one copy of the 406-multiply-add field product for the kernels that add points in a loop
__device__ __noinline__ Fq fq_mul_ni(Fq a, Fq b) { return fq_mul(a, b); }
struct FqMulOutOfLine {
    __device__ Fq operator()(const Fq& a, const Fq& b) const { return fq_mul_ni(a, b); }
};

struct G1A {   // affine, never the identity
    Fq x, y;
};
constexpr int CK_CHUNK = 16;   // table entries per thread of k_ck_tables

// table[(g * windows + k) * digits + d - 1] = d 2^(wbits k) gens[g], affine, digits = 2^wbits - 1.  One thread per
// (g, k, 16 digits): the window's base by doublings, 16 c times the base by double-and-add, then one addition and one
// inversion per entry.
__global__ __launch_bounds__(64) void k_ck_tables(const G1* gens, uint64_t ngens, int windows, int wbits, G1A* table) {
    const uint64_t t = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    const int digits = (1 << wbits) - 1;
    const int chunks = (digits + 1) / CK_CHUNK;
    const uint64_t gk = t / chunks;
    const int chunk = (int)(t % chunks);
    if (gk >= ngens * (uint64_t)windows) return;
    const uint64_t g = gk / windows;
    const int k = (int)(gk % windows);
    const FqMulOutOfLine mul;
    G1 base = gens[g];
#pragma unroll 1
    for (int s = 0; s < wbits * k; ++s) base = g1_dbl_with(base, mul);
    const int first = CK_CHUNK * chunk;
    G1 acc = g1_identity();
#pragma unroll 1
    for (int bit = wbits - 1; bit >= 0; --bit) {
        acc = g1_dbl_with(acc, mul);
        if ((first >> bit) & 1) acc = g1_add_with(acc, base, mul);
    }
    G1A* out = table + gk * (uint64_t)digits;
#pragma unroll 1
    for (int d = first; d < first + CK_CHUNK; ++d) {   // acc = d base
        if (d) {
            const Fq zi = fq_inv_euclid(acc.Z);
            G1A e;
            e.x = fq_mul_ni(acc.X, zi);
            e.y = fq_mul_ni(acc.Y, zi);
            out[d - 1] = e;
        }
        acc = g1_add_with(acc, base, mul);
    }
}

// the product without its conditional subtraction, for the additions without reductions (coordinates below 6q)
__device__ __noinline__ Fq fq_mul_lazy_ni(Fq a, Fq b) { return fq_mul_t<false>(a, b); }
struct FqMulLazyOutOfLine {
    __device__ Fq operator()(const Fq& a, const Fq& b) const { return fq_mul_lazy_ni(a, b); }
};
__device__ inline G1 g1_add_lazy_ni(const G1& p, const G1& q) { return g1_add_lazy_with(p, q, FqMulLazyOutOfLine()); }
__device__ inline G1 g1_add_mixed_lazy_ni(const G1& p, const Fq& x2, const Fq& y2) {
    return g1_add_mixed_lazy_with(p, x2, y2, FqMulLazyOutOfLine());
}

__device__ inline G1 g1_shfl_down(const G1& p, int off) {
    G1 q;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        q.X.v[i] = __shfl_down(p.X.v[i], off, 64);
        q.Y.v[i] = __shfl_down(p.Y.v[i], off, 64);
        q.Z.v[i] = __shfl_down(p.Z.v[i], off, 64);
    }
    return q;
}

constexpr uint32_t CK_QUEUE = 1024;   // ring of digits waiting for a lane: at most 63 left over + 64 x 8 new ones

// One wave per row: sums[row] = rho_row H + sum_c x[row, c] G_c (projective).  The wave reads 64 entries at a time and
// puts their non-zero WB-bit digits (digit, window, sign, column: one word) on a ring in LDS, window by window with
// a ballot and a prefix count; whenever 64 digits wait, every lane takes one and adds its table entry.  Lanes
// therefore never wait for each other's zero digits or shorter entries: a row of n digits costs ceil(n / 64)
// additions per lane.  Lane k < 32 also starts from window k of the blinding scalar.  The 64 partial sums are added
// by a shuffle tree.  The additions skip every reduction: the running sum's coordinates stay below 6q; the table
// entries are affine and below q, so an addition in the loop has eleven products.
template <typename INT, int WB>
__global__ __launch_bounds__(64) void k_commit_rows(const INT* x, uint64_t cols, int windows, const G1A* table,
                                                    const uint32_t* rho_le, const G1A* h_table, G1* sums) {
    static_assert(CK_H_WINDOWS <= 64 && CK_WBITS == 8, "one lane per window (byte) of the blinding scalar");
    constexpr uint32_t DIGITS = (1u << WB) - 1;   // entries per window of the tensor entries' table
    static_assert(WB <= 12, "a queued digit has 12 bits");
    __shared__ uint32_t queue[CK_QUEUE];
    const uint64_t row = blockIdx.x;
    const int lane = threadIdx.x;
    G1 acc = g1_identity();
    if (rho_le) {
        const uint32_t d = lane < CK_H_WINDOWS ? (rho_le[row * 8 + (lane >> 2)] >> (8 * (lane & 3))) & 255u : 0u;
        if (d) {
            const G1A e = h_table[lane * CK_DIGITS + d - 1];
            acc.X = e.x;
            acc.Y = e.y;
            acc.Z = fq_one();
        }
    }
    // one queued digit: acc += (-1)^sign d 2^(WB k) G_c
    auto add_item = [&](uint32_t item) {
        const uint32_t d = item & 0xfffu, k = (item >> 12) & 7u, c = item >> 16;
        const bool negative = (item >> 15) & 1u;
        const G1A e = table[((uint64_t)c * (uint64_t)windows + k) * DIGITS + d - 1];
        const Fq yn = fq_sub2_lazy<2, 1>(fq_zero(), e.y, fq_zero());   // 2q - y: x = r - |x| as a field element is -|x| G
        Fq y2;
#pragma unroll
        for (int i = 0; i < fqc::L; ++i) y2.v[i] = negative ? yn.v[i] : e.y.v[i];
        acc = g1_add_mixed_lazy_ni(acc, e.x, y2);
    };
    const INT* xr = x + row * cols;
    const uint64_t below = ((uint64_t)1 << lane) - 1;   // the lanes before this one
    uint32_t head = 0, tail = 0;                        // the same in every lane
    for (uint64_t c0 = 0; c0 < cols; c0 += 64) {
        const uint64_t c = c0 + (uint64_t)lane;         // below 2^15
        uint64_t mag = 0;
        uint32_t sign = 0;
        if (c < cols) {
            const INT s = xr[c];
            sign = s < 0 ? 1u : 0u;
            mag = sign ? (uint64_t)0 - (uint64_t)(int64_t)s : (uint64_t)s;
        }
        for (int k = 0; k < windows; ++k) {
            if (__ballot(mag != 0) == 0) break;
            const uint32_t d = (uint32_t)mag & DIGITS;
            mag >>= WB;
            const uint64_t has = __ballot(d != 0);
            if (d) queue[(tail + (uint32_t)__popcll(has & below)) % CK_QUEUE] = d | ((uint32_t)k << 12) | (sign << 15) | ((uint32_t)c << 16);
            tail += (uint32_t)__popcll(has);
        }
        __syncthreads();   // one wave: orders the ring's writes before its reads
#pragma unroll 1
        while (tail - head >= 64) {
            add_item(queue[(head + (uint32_t)lane) % CK_QUEUE]);
            head += 64;
        }
    }
    __syncthreads();
    if ((uint32_t)lane < tail - head) add_item(queue[(head + (uint32_t)lane) % CK_QUEUE]);
#pragma unroll 1
    for (int off = 32; off >= 1; off >>= 1) acc = g1_add_lazy_ni(acc, g1_shfl_down(acc, off));
    if (lane == 0) sums[row] = acc;   // coordinates below 6q
}

// affine bytes of the row sums: one inversion per row, one lane per row
__global__ __launch_bounds__(64) void k_commit_affine(const G1* sums, uint64_t rows, uint8_t* out) {
    const uint64_t row = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (row >= rows) return;
    g1_to_bytes(g1_reduce(sums[row]), out + row * 96);
}

// ---- the verifier's side of an opening: two sums of scalar multiples with full field elements as scalars ----
// 96 affine bytes -> Montgomery projective; *ok = false unless both coordinates are below q and the point is on
// the curve (or the bytes are all zero: the identity)
__device__ inline G1 g1_from_bytes(const uint8_t* b, bool* ok) {
    bool all_zero = true;
    for (int i = 0; i < 96; ++i) all_zero = all_zero && b[i] == 0;
    if (all_zero) return g1_identity();
    const Fq xp = fq_limbs_from_bytes(b), yp = fq_limbs_from_bytes(b + 48);
    const Fq q = fq_const(fqc::Q);
    if (!limbs_less(xp, q) || !limbs_less(yp, q)) *ok = false;
    G1 p;
    p.X = fq_to_mont(xp);
    p.Y = fq_to_mont(yp);
    p.Z = fq_one();
    Fq four = fq_add(fq_one(), fq_one());
    four = fq_add(four, four);
    const Fq rhs = fq_add(fq_mul_ni(fq_mul_ni(p.X, p.X), p.X), four);
    if (!fq_eq(fq_mul_ni(p.Y, p.Y), rhs)) *ok = false;
    return p;
}

// ---- a point operation shared by eight lanes -----------------------------------------------------------------
// The complete addition and doubling are two levels of six (four) independent field products with linear steps
// between them.  A group of eight lanes holds the same operands; lane j of the group takes the j-th product of each
// level, the products go round the group by shuffles, and the linear steps are integer combinations of them with
// small coefficients, shifted by a multiple of q so that they stay non-negative, with one carry pass and no
// reduction: the Montgomery product accepts operands up to 2^12 q as long as the limbs are normal.  Coordinates stay
// below 2q between operations (normal limbs); `g1_canonical` reduces them at the end.  An operation is about two
// dependent field products long instead of twelve (eight).
constexpr int COOP = 8;   // lanes per point

// level 1: which coordinates of the first / second operand lane j adds up (bit 0 X, bit 1 Y, bit 2 Z)
__device__ const uint8_t COOP_PICK[2][2][COOP] = {
    {{1, 2, 4, 3, 6, 5, 0, 0}, {1, 2, 4, 3, 6, 5, 0, 0}},    // addition: X1X2, Y1Y2, Z1Z2, (X1+Y1)(X2+Y2), (Y1+Z1)(Y2+Z2), (X1+Z1)(X2+Z2)
    {{2, 2, 4, 1, 0, 0, 0, 0}, {2, 4, 4, 2, 0, 0, 0, 0}}};   // doubling: Y Y, Y Z, Z Z, X Y
// level 2: the two operands of lane j as combinations of the six level-1 products, last entry: multiples of q
//   addition (T = t0, t1, t2, p3, p4, p5):  t3 = p3 - t0 - t1, t4 = p4 - t1 - t2, y3 = 12 (p5 - t0 - t2),
//     t1' = t1 - 12 t2, z3 = t1 + 12 t2, x3 = 3 t0;  products t4 y3, t3 t1', y3 x3, t1' z3, x3 t3, z3 t4
//   doubling (T = Y^2, YZ, Z^2, XY):  products (12 Z^2)(8 Y^2), (YZ)(8 Y^2), (Y^2 - 36 Z^2)(Y^2 + 12 Z^2), (Y^2 - 36 Z^2)(XY)
__device__ const int8_t COOP_LIN[2][COOP][2][7] = {
    {{{0, -1, -1, 0, 1, 0, 2}, {-12, 0, -12, 0, 0, 12, 24}},
     {{-1, -1, 0, 1, 0, 0, 2}, {0, 1, -12, 0, 0, 0, 12}},
     {{-12, 0, -12, 0, 0, 12, 24}, {3, 0, 0, 0, 0, 0, 0}},
     {{0, 1, -12, 0, 0, 0, 12}, {0, 1, 12, 0, 0, 0, 0}},
     {{3, 0, 0, 0, 0, 0, 0}, {-1, -1, 0, 1, 0, 0, 2}},
     {{0, 1, 12, 0, 0, 0, 0}, {0, -1, -1, 0, 1, 0, 2}},
     {{0, 0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0, 0}},
     {{0, 0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0, 0}}},
    {{{0, 0, 12, 0, 0, 0, 0}, {8, 0, 0, 0, 0, 0, 0}},
     {{0, 1, 0, 0, 0, 0, 0}, {8, 0, 0, 0, 0, 0, 0}},
     {{1, 0, -36, 0, 0, 0, 36}, {1, 0, 12, 0, 0, 0, 0}},
     {{1, 0, -36, 0, 0, 0, 36}, {0, 0, 0, 1, 0, 0, 0}},
     {{0, 0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0, 0}},
     {{0, 0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0, 0}},
     {{0, 0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0, 0}},
     {{0, 0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0, 0}}}};

__device__ inline Fq coop_pick(const G1& p, uint32_t sel) {
    const uint32_t mx = 0u - (sel & 1u), my = 0u - ((sel >> 1) & 1u), mz = 0u - ((sel >> 2) & 1u);
    Fq o;
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        const uint32_t x = (p.X.v[i] & mx) + (p.Y.v[i] & my) + (p.Z.v[i] & mz) + c;
        o.v[i] = i < fqc::L - 1 ? (x & fqc::M29) : x;
        c = i < fqc::L - 1 ? (x >> 29) : 0;
    }
    return o;
}

// sum_s c[s] T[s] + c[6] q, carried into normal limbs (the caller's coefficients keep it in [0, 2^12 q))
__device__ inline Fq coop_lin(const Fq (&T)[6], const int (&c)[7]) {
    Fq o;
    int64_t acc = 0;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        acc += (int64_t)c[6] * (int64_t)fqc::Q[i];
#pragma unroll
        for (int s = 0; s < 6; ++s) acc += (int64_t)c[s] * (int64_t)T[s].v[i];
        o.v[i] = i < fqc::L - 1 ? ((uint32_t)acc & fqc::M29) : (uint32_t)acc;
        acc >>= 29;
    }
    return o;
}

__device__ inline void coop_gather(const Fq& mine, Fq (&T)[6]) {
#pragma unroll
    for (int s = 0; s < 6; ++s)
#pragma unroll
        for (int i = 0; i < fqc::L; ++i) T[s].v[i] = __shfl(mine.v[i], s, COOP);
}

// MODE 0: p + q, MODE 1: 2 p (q is not read).  Every lane of the group passes the same operands and gets the same
// result; all 64 lanes of the wave must call it together.
template <int MODE>
__device__ inline G1 g1_coop(const G1& p, const G1& q, int j) {
    Fq T[6];
    coop_gather(fq_mul_ni(coop_pick(p, COOP_PICK[MODE][0][j]), coop_pick(MODE ? p : q, COOP_PICK[MODE][1][j])), T);
    int ca[7], cb[7];
#pragma unroll
    for (int s = 0; s < 7; ++s) {
        ca[s] = COOP_LIN[MODE][j][0][s];
        cb[s] = COOP_LIN[MODE][j][1][s];
    }
    coop_gather(fq_mul_ni(coop_lin(T, ca), coop_lin(T, cb)), T);
    G1 r;
    if (MODE == 0) {
        const int cx[7] = {-1, 1, 0, 0, 0, 0, 1}, cy[7] = {0, 0, 1, 1, 0, 0, 0}, cz[7] = {0, 0, 0, 0, 1, 1, 0};
        r.X = coop_lin(T, cx);
        r.Y = coop_lin(T, cy);
        r.Z = coop_lin(T, cz);
    } else {
        const int cx[7] = {0, 0, 0, 2, 0, 0, 0}, cy[7] = {1, 0, 1, 0, 0, 0, 0};
        r.X = coop_lin(T, cx);
        r.Y = coop_lin(T, cy);
        r.Z = T[1];
    }
    return r;
}

__device__ inline G1 g1_canonical(const G1& p) {   // coordinates below 2q -> below q
    G1 r;
    r.X = fq_cond_sub(p.X);
    r.Y = fq_cond_sub(p.Y);
    r.Z = fq_cond_sub(p.Z);
    return r;
}

constexpr int MSM_TERMS = 64 / COOP;   // terms per block
constexpr int G1_WORDS = 3 * fqc::L;

// |z| for the curve's parameter z = -0xd201000000010000: r = z^4 - z^2 + 1 = (-z^2)^2 + (-z^2) + 1, so -z^2 is a
// cube root of unity modulo r.  The map phi(x, y) = (beta x, y), beta a cube root of unity in F_q, is an
// endomorphism of the curve; on the subgroup of order r it is multiplication by a cube root of unity modulo r, and
// beta is chosen (on the host, by trying both roots on a subgroup point: endo_beta) so that phi(P) = -z^2 P there.
constexpr uint64_t CK_Z_ABS = 0xd201000000010000ull;

// |z| p for a group of eight lanes: the top bit of |z| is bit 63
__device__ inline G1 coop_mul_zabs(const G1& p, int j) {
    G1 acc = p;
#pragma unroll 1
    for (int bit = 62; bit >= 0; --bit) {
        acc = g1_coop<1>(acc, acc, j);
        if ((CK_Z_ABS >> bit) & 1ull) acc = g1_coop<0>(acc, p, j);   // the same branch in every lane
    }
    return acc;
}

// Eight lanes per term of two sums in one launch: the blocks below nb_bytes take the points given as affine bytes
// (term t = 8 block + group < n_bytes, scalar scal[t]), the next nb_g1 blocks the key's generators (term t' = 8
// (block - nb_bytes) + group < n_g1, scalar scal[n_bytes + t']).  A scalar k < r comes split as k = a + b z^2 with
// a, b < 2^128 (4 + 4 words, little-endian), so that k P = a P + b (-phi(P)) for P in the subgroup: half as many
// doublings.  A group first builds the 15 multiples of its point and their images (beta X, -Y, Z) in LDS, then runs
// over the 32 4-bit windows from the top: four doublings and two additions of table entries (of the identity for a
// zero digit: the formulas are complete, and the wave stays in step).  Three more additions sum the block's terms:
// part[block], coordinates below 2q.
// The last nb_bytes blocks check that the points given as bytes are elements of the subgroup, for which the split
// holds and in which Sec. 2.3 works: phi(P) = -z^2 P exactly when r P = O (if phi(P) = -z^2 P then
// (z^4 - z^2 + 1) P = (phi^2 + phi + 1) P = O; conversely phi acts on the subgroup as the root -z^2 by the choice
// of beta), at the cost of 126 doublings and 10 additions next to the sums' 128 doublings.
// bad[0] is set if a point given as bytes is malformed or outside the subgroup.
__global__ __launch_bounds__(64) void k_msm_terms(const uint8_t* pts_bytes, uint64_t n_bytes, unsigned nb_bytes,
                                                  const G1* pts_g1, uint64_t n_g1, unsigned nb_g1, const uint32_t* scal,
                                                  G1* part, uint32_t* bad, Fq beta) {
    __shared__ uint32_t tab[2][MSM_TERMS][15][G1_WORDS];
    const int j = threadIdx.x % COOP, grp = threadIdx.x / COOP;
    if (blockIdx.x >= nb_bytes + nb_g1) {   // subgroup check of eight of the points given as bytes
        const uint64_t t = (blockIdx.x - nb_bytes - nb_g1) * (uint64_t)MSM_TERMS + grp;
        const bool live = t < n_bytes;
        bool ok = true;
        const G1 p = live ? g1_from_bytes(pts_bytes + 96 * t, &ok) : g1_identity();
        const G1 zz = coop_mul_zabs(coop_mul_zabs(p, j), j);   // z^2 P
        if (live && j == 0 && !fq_is_zero(p.Z)) {              // P affine: beta x Z' = X' and y Z' = -Y'
            const Fq zc = fq_cond_sub(zz.Z);
            ok = ok && fq_eq(fq_mul_ni(fq_mul_ni(beta, p.X), zc), fq_cond_sub(zz.X));
            ok = ok && fq_is_zero(fq_add(fq_mul_ni(p.Y, zc), fq_cond_sub(zz.Y)));
            if (!ok) bad[0] = 1;
        }
        return;
    }
    const bool from_bytes = blockIdx.x < nb_bytes;
    const uint64_t t = (from_bytes ? blockIdx.x : blockIdx.x - nb_bytes) * (uint64_t)MSM_TERMS + grp;
    const bool live = t < (from_bytes ? n_bytes : n_g1);
    G1 base = g1_identity();
    uint32_t k[8];
#pragma unroll
    for (int w = 0; w < 8; ++w) k[w] = 0;
    if (live) {
        bool ok = true;
        base = from_bytes ? g1_from_bytes(pts_bytes + 96 * t, &ok) : pts_g1[t];
        if (!ok) bad[0] = 1;
        const uint32_t* sp = scal + 8 * (from_bytes ? t : n_bytes + t);
#pragma unroll
        for (int w = 0; w < 8; ++w) k[w] = sp[w];
    }
    G1 acc = base;
#pragma unroll 1
    for (int d = 0; d < 15; ++d) {   // tab[0][d] = (d + 1) base, tab[1][d] = -phi of it
        if (d) acc = g1_coop<0>(acc, base, j);
        const Fq bx = fq_mul_ni(acc.X, beta);
        const Fq ny = fq_neg(fq_cond_sub(acc.Y));
        if (j == 0) {
#pragma unroll
            for (int i = 0; i < fqc::L; ++i) {
                tab[0][grp][d][i] = acc.X.v[i];
                tab[0][grp][d][fqc::L + i] = acc.Y.v[i];
                tab[0][grp][d][2 * fqc::L + i] = acc.Z.v[i];
                tab[1][grp][d][i] = bx.v[i];
                tab[1][grp][d][fqc::L + i] = ny.v[i];
                tab[1][grp][d][2 * fqc::L + i] = acc.Z.v[i];
            }
        }
    }
    __syncthreads();
    acc = g1_identity();
#pragma unroll 1
    for (int win = 31; win >= 0; --win) {
#pragma unroll 1
        for (int q = 0; q < 4; ++q) acc = g1_coop<1>(acc, acc, j);
#pragma unroll 1
        for (int half = 0; half < 2; ++half) {
            const uint32_t dg = (k[4 * half + (win >> 3)] >> (4 * (win & 7))) & 15u;
            G1 e = g1_identity();
            if (dg) {
                const uint32_t* src = tab[half][grp][dg - 1];
#pragma unroll
                for (int i = 0; i < fqc::L; ++i) {
                    e.X.v[i] = src[i];
                    e.Y.v[i] = src[fqc::L + i];
                    e.Z.v[i] = src[2 * fqc::L + i];
                }
            }
            acc = g1_coop<0>(acc, e, j);
        }
    }
#pragma unroll 1
    for (int off = 32; off >= COOP; off >>= 1) acc = g1_coop<0>(acc, g1_shfl_down(acc, off), j);
    if (threadIdx.x == 0) part[blockIdx.x] = acc;
}

// Block b: the sum of part[first[b] .. first[b] + count[b]) (coordinates below 2q): one wave, eight groups of lanes
// adding every eighth partial sum, three more additions; then either its affine bytes at out + 96 b (one inversion)
// or, with proj != nullptr, the projective sum itself at proj[b], coordinates below q (the caller compares two sums
// by cross-multiplication and needs no inversion).
__global__ __launch_bounds__(64) void k_msm_finish(const G1* part, uint64_t n0, uint64_t n1, uint8_t* out, G1* proj) {
    const int j = threadIdx.x % COOP, grp = threadIdx.x / COOP;
    const G1* src = blockIdx.x ? part + n0 : part;
    const uint64_t n = blockIdx.x ? n1 : n0;
    G1 acc = g1_identity();
#pragma unroll 1
    for (uint64_t i = 0; i < n; i += MSM_TERMS) {   // every group runs the same number of trips
        const uint64_t at = i + grp;
        const G1 e = at < n ? src[at] : g1_identity();
        acc = g1_coop<0>(acc, e, j);
    }
#pragma unroll 1
    for (int off = 32; off >= COOP; off >>= 1) acc = g1_coop<0>(acc, g1_shfl_down(acc, off), j);
    if (threadIdx.x == 0) {
        if (proj) proj[blockIdx.x] = g1_canonical(acc);
        else g1_to_bytes(g1_canonical(acc), out + 96 * blockIdx.x);
    }
}

__global__ __launch_bounds__(64) void k_ck_export(const G1* gens, uint64_t first, uint64_t count, uint8_t* out) {
    const uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (i >= count) return;
    g1_to_bytes(gens[first + i], out + i * 96);
}

}  // namespace

struct zkdl_commit_key {
    uint64_t ncols;
    int max_bits;     // widest tensor entry served: 32 or 64
    int wbits;        // bits per window of a tensor entry: 8 or 12
    int windows;      // windows of a tensor entry: max_bits / wbits, rounded up
    G1* gens;         // device: ncols generators, then H
    G1A* table;       // device: [ncols][windows][2^wbits - 1], affine
    G1A* h_table;     // device: [32][255]
};

// ---- host: the endomorphism's constant and the split of a scalar -------------------------------------------------
// a point of the curve found by trying x = 1, 2, .. (Montgomery form, Z = 1)
static bool host_curve_point(G1* out) {
    Fq xs = fq_zero();
    const Fq four = fq_add(fq_add(fq_one(), fq_one()), fq_add(fq_one(), fq_one()));
    for (int t = 0; t < 64; ++t) {
        xs = fq_add(xs, fq_one());
        const Fq rhs = fq_add(fq_mul(fq_sqr(xs), xs), four);
        const Fq y = fq_pow(rhs, fqc::EXP_SQRT);
        if (fq_eq(fq_sqr(y), rhs) && !fq_is_zero(y)) {
            out->X = xs;
            out->Y = y;
            out->Z = fq_one();
            return true;
        }
    }
    return false;
}

// beta with phi(P) = (beta x, y) = -z^2 P on the subgroup: beta = (-1 +- sqrt(-3)) / 2, the sign found by trying both
// on a point that the cofactor has taken into the subgroup.  false if neither fits (a broken constant).
static bool make_endo_beta(Fq* beta) {
    const Fq one = fq_one(), two = fq_add(one, one), m3 = fq_neg(fq_add(two, one));
    const Fq s = fq_pow(m3, fqc::EXP_SQRT);
    if (!fq_eq(fq_sqr(s), m3)) return false;
    const Fq half = fq_inv_euclid(two);
    const Fq cand[2] = {fq_mul(fq_sub(s, one), half), fq_mul(fq_sub(fq_neg(s), one), half)};
    G1 p0;
    if (!host_curve_point(&p0)) return false;
    const G1 p = g1_mul_words(p0, fqc::COFACTOR);
    if (fq_is_zero(p.Z)) return false;
    const uint32_t zw[2] = {(uint32_t)CK_Z_ABS, (uint32_t)(CK_Z_ABS >> 32)};
    const G1 q = g1_mul_words(g1_mul_words(p, zw), zw);   // z^2 P
    for (int c = 0; c < 2; ++c) {
        const bool x_fits = fq_eq(fq_mul(fq_mul(cand[c], p.X), q.Z), fq_mul(q.X, p.Z));
        const bool y_fits = fq_is_zero(fq_add(fq_mul(p.Y, q.Z), fq_mul(q.Y, p.Z)));
        if (x_fits && y_fits && !fq_eq(cand[c], one) && fq_eq(fq_mul(fq_sqr(cand[c]), cand[c]), one)) {
            *beta = cand[c];
            return true;
        }
    }
    return false;
}

static bool endo_beta(Fq* beta) {
    static Fq value;
    static const bool ok = make_endo_beta(&value);
    *beta = value;
    return ok;
}

// k = a + b z^2 with a < z^2: out[0..3] = a, out[4..7] = b (32-bit words, least significant first); false unless
// b < 2^128 (true for every k < r < z^4).  Long division in base 2^32 (Knuth, Algorithm D; the divisor's top bit
// is set, so nothing is shifted), and the result is multiplied out again before it is trusted.
static bool glv_split(const uint32_t k[8], uint32_t out[8]) {
    const unsigned __int128 zz = (unsigned __int128)CK_Z_ABS * CK_Z_ABS;
    uint32_t v[4], un[9], q[5];
    for (int i = 0; i < 4; ++i) v[i] = (uint32_t)(zz >> (32 * i));
    for (int i = 0; i < 8; ++i) un[i] = k[i];
    un[8] = 0;
    for (int jj = 4; jj >= 0; --jj) {
        const uint64_t num = ((uint64_t)un[jj + 4] << 32) | un[jj + 3];
        uint64_t qhat = num / v[3], rhat = num % v[3];
        while (qhat >> 32 || qhat * v[2] > ((rhat << 32) | un[jj + 2])) {
            --qhat;
            rhat += v[3];
            if (rhat >> 32) break;
        }
        uint64_t carry = 0;
        int64_t borrow = 0;
        for (int i = 0; i < 4; ++i) {
            const uint64_t prod = qhat * v[i] + carry;
            carry = prod >> 32;
            const int64_t d = (int64_t)un[jj + i] - (int64_t)(uint32_t)prod - borrow;
            un[jj + i] = (uint32_t)d;
            borrow = d < 0 ? 1 : 0;
        }
        const int64_t d = (int64_t)un[jj + 4] - (int64_t)carry - borrow;
        un[jj + 4] = (uint32_t)d;
        if (d < 0) {   // the estimate was one too large: add the divisor back
            --qhat;
            uint64_t c = 0;
            for (int i = 0; i < 4; ++i) {
                c += (uint64_t)un[jj + i] + v[i];
                un[jj + i] = (uint32_t)c;
                c >>= 32;
            }
            un[jj + 4] += (uint32_t)c;
        }
        q[jj] = (uint32_t)qhat;
    }
    if (q[4] != 0) return false;
    unsigned __int128 a = 0, b = 0;
    for (int i = 3; i >= 0; --i) {
        a = (a << 32) | un[i];
        b = (b << 32) | q[i];
        out[i] = un[i];
        out[4 + i] = q[i];
    }
    if (a >= zz || un[4] || un[5] || un[6] || un[7]) return false;
    // a + b z^2 = k, multiplied out in 32-bit words
    uint32_t back[9] = {0};
    for (int i = 0; i < 4; ++i) {
        uint64_t c = 0;
        for (int l = 0; l < 4; ++l) {
            c += (uint64_t)q[i] * v[l] + back[i + l];
            back[i + l] = (uint32_t)c;
            c >>= 32;
        }
        back[i + 4] += (uint32_t)c;
    }
    uint64_t c = 0;
    for (int i = 0; i < 8; ++i) {
        c += (uint64_t)back[i] + (i < 4 ? un[i] : 0u);
        if ((uint32_t)c != k[i]) return false;
        c >>= 32;
    }
    return c == 0;
}

extern "C" int zkdl_host_scalar_split(const zkdl_fr* k, uint8_t out[32]) {
    if (!k || !out) return ZKDL_EINVAL;
    uint32_t kw[8], ab[8];
    memcpy(kw, k->le, 32);
    if (!glv_split(kw, ab)) return ZKDL_EINVAL;
    memcpy(out, ab, 32);
    return ZKDL_OK;
}

// host-side check of the constants of fq.cuh (no GPU needed): Montgomery one and R^2 by repeated doubling,
// the Montgomery factor, the square-root and inversion exponents
static int commit_selfcheck_run() {
    Fq x = fq_zero();
    x.v[0] = 1;
    for (int i = 0; i < 406; ++i) x = fq_add(x, x);
    if (!fq_eq(x, fq_const(fqc::ONE))) return ZKDL_EINVAL;
    for (int i = 0; i < 406; ++i) x = fq_add(x, x);
    if (!fq_eq(x, fq_const(fqc::R2))) return ZKDL_EINVAL;
    if (((fqc::Q[0] * fqc::NINV) & fqc::M29) != fqc::M29) return ZKDL_EINVAL;   // q * (-q^{-1}) = -1 mod 2^29
    // 3^(q-2) * 3 = 1 and (3^2)^((q+1)/4) = +-3
    Fq three = fq_add(fq_one(), fq_add(fq_one(), fq_one()));
    if (!fq_eq(fq_mul(fq_inv(three), three), fq_one())) return ZKDL_EINVAL;
    Fq root = fq_pow(fq_sqr(three), fqc::EXP_SQRT);
    if (!fq_eq(root, three) && !fq_eq(root, fq_neg(three))) return ZKDL_EINVAL;
    // the Euclidean inversion against a^(q-2): limb values 1, 2, q - 1, 2^380, then a chain of products
    Fq probe[16];
    probe[0] = fq_zero();
    probe[0].v[0] = 1;
    probe[1] = fq_add(probe[0], probe[0]);
    probe[2] = fq_sub(fq_zero(), probe[0]);
    probe[3] = fq_zero();
    probe[3].v[13] = 1u << 3;
    probe[4] = fq_one();
    probe[5] = fq_neg(fq_one());
    for (int i = 6; i < 16; ++i) probe[i] = fq_add(fq_mul(probe[i - 1], fq_add(three, probe[i - 3])), probe[i - 2]);
    for (int i = 0; i < 16; ++i)
        if (!fq_eq(fq_inv_euclid(probe[i]), fq_inv(probe[i]))) return ZKDL_EINVAL;
    if (!fq_is_zero(fq_inv_euclid(fq_zero()))) return ZKDL_EINVAL;
    // the additions without reductions against the reduced one, on multiples of a point found by trying x = 1, 2, ..:
    // a running sum that only ever goes through the lazy forms (so its coordinates take the bounds the kernel's do),
    // the sum from the identity, a point added to itself and to its negative
    G1 base;
    if (!host_curve_point(&base)) return ZKDL_EINVAL;
    auto same = [](const G1& a, const G1& b) {   // equal as projective points, coordinates reduced
        return fq_eq(fq_mul(a.X, b.Z), fq_mul(b.X, a.Z)) && fq_eq(fq_mul(a.Y, b.Z), fq_mul(b.Y, a.Z)) &&
               fq_is_zero(a.Z) == fq_is_zero(b.Z);
    };
    auto affine = [](const G1& p, Fq* x, Fq* y) {
        const Fq zi = fq_inv_euclid(p.Z);
        *x = fq_mul(p.X, zi);
        *y = fq_mul(p.Y, zi);
    };
    const FqMulLazyInline lazy;
    G1 term = base, sum = g1_identity(), lsum = g1_identity(), msum = g1_identity();
    for (int i = 0; i < 40; ++i) {
        Fq tx, ty;
        affine(term, &tx, &ty);
        Fq y2 = ty;
        if (i % 3 == 1) {   // every third term negated the way the kernel negates (2q - y)
            term = g1_neg(term);
            y2 = fq_sub2_lazy<2, 1>(fq_zero(), ty, fq_zero());
        }
        sum = g1_add(sum, term);
        lsum = g1_add_lazy_with(lsum, term, lazy);
        msum = g1_add_mixed_lazy_with(msum, tx, y2, lazy);
        if (!same(g1_reduce(lsum), sum) || !same(g1_reduce(msum), sum)) return ZKDL_EINVAL;
        if (!same(g1_reduce(g1_add_lazy_with(lsum, msum, lazy)), g1_dbl(sum))) return ZKDL_EINVAL;   // two lazy operands
        term = g1_add(g1_dbl(term), base);
    }
    {
        Fq bx, by;
        affine(base, &bx, &by);
        const Fq byn = fq_sub2_lazy<2, 1>(fq_zero(), by, fq_zero());
        if (!same(g1_reduce(g1_add_mixed_lazy_with(base, bx, by, lazy)), g1_dbl(base))) return ZKDL_EINVAL;
        const G1 o = g1_reduce(g1_add_mixed_lazy_with(base, bx, byn, lazy));
        if (!fq_is_zero(o.Z) || !fq_is_zero(o.X)) return ZKDL_EINVAL;
        const G1 o2 = g1_reduce(g1_add_lazy_with(base, g1_neg(base), lazy));
        if (!fq_is_zero(o2.Z) || !fq_is_zero(o2.X)) return ZKDL_EINVAL;
    }
    // the endomorphism: its constant, and the split of a scalar on edge values (0, 1, z^2 - 1, z^2, z^2 + 1, r - 1,
    // 2^256 - 1 is refused) and on a chain of mixed words; with the split, k P = a P + b (-phi(P)) on a subgroup point
    Fq beta;
    if (!endo_beta(&beta)) return ZKDL_EINVAL;
    {
        const unsigned __int128 zz = (unsigned __int128)CK_Z_ABS * CK_Z_ABS;
        uint32_t ks[8][8] = {};
        ks[1][0] = 1;
        for (int i = 0; i < 4; ++i) {
            ks[2][i] = (uint32_t)((zz - 1) >> (32 * i));
            ks[3][i] = (uint32_t)(zz >> (32 * i));
            ks[4][i] = (uint32_t)((zz + 1) >> (32 * i));
        }
        for (int i = 0; i < 8; ++i) ks[5][i] = frc::MOD[i];
        ks[5][0] -= 1;
        uint32_t w = 0x9e3779b9u;
        for (int i = 0; i < 8; ++i) {
            w = w * 1664525u + 1013904223u;
            ks[6][i] = i == 7 ? (w & 0x3fffffffu) : w;
            ks[7][i] = i == 7 ? 0x73eda752u : ~w;
        }
        const G1 p = g1_mul_words(base, fqc::COFACTOR);   // in the subgroup
        G1 nphi = p;                                      // -phi(P) = (beta X, -Y, Z)
        nphi.X = fq_mul(p.X, beta);
        nphi.Y = fq_neg(p.Y);
        for (int t = 0; t < 8; ++t) {
            uint32_t ab[8];
            if (!glv_split(ks[t], ab)) return ZKDL_EINVAL;
            const uint32_t a4[4] = {ab[0], ab[1], ab[2], ab[3]}, b4[4] = {ab[4], ab[5], ab[6], ab[7]};
            if (t >= 5 && !same(g1_mul_words(p, ks[t]), g1_add(g1_mul_words(p, a4), g1_mul_words(nphi, b4))))
                return ZKDL_EINVAL;
        }
        uint32_t all_ones[8], ab[8];
        for (int i = 0; i < 8; ++i) all_ones[i] = 0xffffffffu;
        if (glv_split(all_ones, ab)) return ZKDL_EINVAL;   // the quotient does not fit 128 bits
        // a point outside the subgroup does not pass the membership test phi(P) = -z^2 P
        const uint32_t zw[2] = {(uint32_t)CK_Z_ABS, (uint32_t)(CK_Z_ABS >> 32)};
        const G1 q = g1_mul_words(g1_mul_words(base, zw), zw);
        const bool base_in = fq_is_zero(g1_mul_words(base, frc::MOD).Z);
        const bool passes = fq_eq(fq_mul(fq_mul(beta, base.X), q.Z), fq_mul(q.X, base.Z)) &&
                            fq_is_zero(fq_add(fq_mul(base.Y, q.Z), fq_mul(q.Y, base.Z)));
        if (base_in != passes) return ZKDL_EINVAL;
    }
    return ZKDL_OK;
}

// the checks run once per process: they take some milliseconds of host arithmetic
extern "C" int zkdl_commit_selfcheck(void) {
    static const int rc = commit_selfcheck_run();
    return rc;
}

extern "C" int zkdl_commit_key_destroy(zkdl_ctx* ctx, zkdl_commit_key* key) {
    if (!ctx || !key) return ZKDL_EINVAL;
    (void)hipStreamSynchronize(ctx->stream);
    zk_free(ctx, key->gens);
    zk_free(ctx, key->table);
    zk_free(ctx, key->h_table);
    delete key;
    return ZKDL_OK;
}

extern "C" int zkdl_commit_key_create(zkdl_ctx* ctx, const char* label, uint64_t ncols, int max_bits,
                                      zkdl_commit_key** out) {
    if (!ctx || !label || !out || (max_bits != 32 && max_bits != 64)) return ZKDL_EINVAL;
    const size_t ll = strlen(label);
    if (ll > (size_t)CK_MAX_LABEL || ncols == 0 || (ncols & (ncols - 1)) || ncols > ((uint64_t)1 << 15)) return ZKDL_EINVAL;
    if (zkdl_commit_selfcheck() != ZKDL_OK) return ZKDL_EINVAL;
    ZK_HIP(ctx, hipSetDevice(ctx->device));
    zkdl_commit_key* key = new (std::nothrow) zkdl_commit_key();
    if (!key) return ZKDL_ENOMEM;
    key->ncols = ncols;
    key->max_bits = max_bits;
    // wide windows save additions (a 32-bit entry has three 12-bit digits instead of four bytes, a 12-bit one a single
    // digit) and cost 16 times the entries per window: taken while the tables stay a small part of the memory
    const uint64_t wide_bytes = sizeof(G1A) * ncols * (uint64_t)((max_bits + CK_WIDE_WBITS - 1) / CK_WIDE_WBITS) *
                                (((uint64_t)1 << CK_WIDE_WBITS) - 1);
    key->wbits = ctx->commit_wbits ? ctx->commit_wbits : (wide_bytes <= CK_WIDE_MAX_BYTES ? CK_WIDE_WBITS : CK_WBITS);
    key->windows = (max_bits + key->wbits - 1) / key->wbits;
    const uint64_t digits = ((uint64_t)1 << key->wbits) - 1;
    key->gens = (G1*)zk_alloc(ctx, sizeof(G1) * (ncols + 1));
    key->table = (G1A*)zk_alloc(ctx, sizeof(G1A) * ncols * key->windows * digits);
    key->h_table = (G1A*)zk_alloc(ctx, sizeof(G1A) * CK_H_WINDOWS * CK_DIGITS);
    if (!key->gens || !key->table || !key->h_table) {
        zkdl_commit_key_destroy(ctx, key);
        return ZKDL_ENOMEM;
    }
    LabelArg la;
    memcpy(la.bytes, "zkdl-mi355x/g1/", 15);
    memcpy(la.bytes + 15, label, ll);
    la.len = (uint32_t)(15 + ll);
    const Fq r2x = r2x_const();
    hipLaunchKernelGGL(k_ck_generators, dim3((unsigned)((ncols + 1 + 63) / 64)), dim3(64), 0, ctx->stream, la, ncols,
                       key->gens, r2x);
    // threads per (generator, window): a 16th of the entries
    const uint64_t nt = ncols * key->windows * ((digits + 1) / CK_CHUNK);
    const uint64_t nh = (uint64_t)CK_H_WINDOWS * ((CK_DIGITS + 1) / CK_CHUNK);
    hipLaunchKernelGGL(k_ck_tables, dim3((unsigned)((nt + 63) / 64)), dim3(64), 0, ctx->stream, key->gens, ncols,
                       key->windows, key->wbits, key->table);
    hipLaunchKernelGGL(k_ck_tables, dim3((unsigned)((nh + 63) / 64)), dim3(64), 0, ctx->stream, key->gens + ncols,
                       (uint64_t)1, CK_H_WINDOWS, CK_WBITS, key->h_table);
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) {
        ctx->last_hip = (int)e;
        zkdl_commit_key_destroy(ctx, key);
        return ZKDL_EHIP;
    }
    *out = key;
    return ZKDL_OK;
}

extern "C" int zkdl_commit_key_generators(zkdl_ctx* ctx, const zkdl_commit_key* key, uint64_t first, uint64_t count,
                                          uint8_t* host_out) {
    if (!ctx || !key || !host_out || first + count > key->ncols + 1 || count == 0) return ZKDL_EINVAL;
    uint8_t* dev = (uint8_t*)zk_alloc(ctx, count * 96);
    if (!dev) return ZKDL_ENOMEM;
    hipLaunchKernelGGL(k_ck_export, dim3((unsigned)((count + 63) / 64)), dim3(64), 0, ctx->stream, key->gens, first, count, dev);
    hipError_t e = hipMemcpyAsync(host_out, dev, count * 96, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    zk_free(ctx, dev);
    ZK_HIP(ctx, e);
    return ZKDL_OK;
}

extern "C" int hyrax_commit(zkdl_ctx* ctx, const zkdl_commit_key* key, const zkdl_tensor* X, const zkdl_fr* blind,
                            uint8_t* commitments_out, size_t* ncommit) {
    if (!ctx || !key || !X || !commitments_out || !ncommit) return ZKDL_EINVAL;
    if (X->kind != TK_I32 && X->kind != TK_I64) return ZKDL_EINVAL;
    if (X->kind == TK_I64 && key->max_bits < 64) return ZKDL_EINVAL;
    int m = 0;
    while (((uint64_t)1 << m) < X->numel) ++m;
    if (((uint64_t)1 << m) != X->numel) return ZKDL_EINVAL;
    const uint64_t cols = (uint64_t)1 << (m / 2), rows = (uint64_t)1 << (m - m / 2);
    if (cols > key->ncols) return ZKDL_EINVAL;
    if (*ncommit < rows) {
        *ncommit = rows;
        return ZKDL_ESMALL;
    }
    for (uint64_t j = 0; blind && j < rows; ++j) {   // blinding scalars are field elements: below r
        bool below = false;
        for (int i = 31; i >= 0 && !below; --i) {
            const uint8_t rb = (uint8_t)(frc::MOD[i >> 2] >> (8 * (i & 3)));
            if (blind[j].le[i] > rb) return ZKDL_EINVAL;
            below = blind[j].le[i] < rb;
        }
        if (!below) return ZKDL_EINVAL;
    }
    ZK_HIP(ctx, hipSetDevice(ctx->device));
    G1* part = (G1*)zk_alloc(ctx, sizeof(G1) * rows);
    uint8_t* out_dev = (uint8_t*)zk_alloc(ctx, rows * 96);
    uint32_t* rho_dev = blind ? (uint32_t*)zk_alloc(ctx, rows * 32) : nullptr;
    int rc = (part && out_dev && (!blind || rho_dev)) ? ZKDL_OK : ZKDL_ENOMEM;
    hipError_t e = hipSuccess;
    if (rc == ZKDL_OK && blind) e = hipMemcpyAsync(rho_dev, blind, rows * 32, hipMemcpyHostToDevice, ctx->stream);
    if (rc == ZKDL_OK && e == hipSuccess) {
        // the key's tables have `windows` entries per generator whatever the tensor's width
        const dim3 grid((unsigned)rows), block(64);
        if (X->kind == TK_I32 && key->wbits == CK_WIDE_WBITS)
            hipLaunchKernelGGL((k_commit_rows<int32_t, CK_WIDE_WBITS>), grid, block, 0, ctx->stream,
                               (const int32_t*)X->data, cols, key->windows, key->table, rho_dev, key->h_table, part);
        else if (X->kind == TK_I32)
            hipLaunchKernelGGL((k_commit_rows<int32_t, CK_WBITS>), grid, block, 0, ctx->stream,
                               (const int32_t*)X->data, cols, key->windows, key->table, rho_dev, key->h_table, part);
        else if (key->wbits == CK_WIDE_WBITS)
            hipLaunchKernelGGL((k_commit_rows<int64_t, CK_WIDE_WBITS>), grid, block, 0, ctx->stream,
                               (const int64_t*)X->data, cols, key->windows, key->table, rho_dev, key->h_table, part);
        else
            hipLaunchKernelGGL((k_commit_rows<int64_t, CK_WBITS>), grid, block, 0, ctx->stream,
                               (const int64_t*)X->data, cols, key->windows, key->table, rho_dev, key->h_table, part);
        hipLaunchKernelGGL(k_commit_affine, dim3((unsigned)((rows + 63) / 64)), dim3(64), 0, ctx->stream, part, rows, out_dev);
        e = hipMemcpyAsync(commitments_out, out_dev, rows * 96, hipMemcpyDeviceToHost, ctx->stream);
    }
    hipError_t e2 = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess) e = e2;
    if (e == hipSuccess) e = hipGetLastError();
    zk_free(ctx, part);
    zk_free(ctx, out_dev);
    zk_free(ctx, rho_dev);
    if (rc != ZKDL_OK) return rc;
    ZK_HIP(ctx, e);
    *ncommit = rows;
    return ZKDL_OK;
}

// host: beta~(u, .) over 2^m entries (Montgomery form), u canonical bytes
static bool host_beta_table(const zkdl_fr* u, int m, std::vector<Fr>& out) {
    out.assign((size_t)1 << m, fr_zero());
    out[0] = fr_one();
    size_t size = 1;
    for (int k = m - 1; k >= 0; --k) {   // coordinate 0 pairs with the most significant bit
        Fr x;
        memcpy(x.v, u[k].le, 32);
        bool below = false;
        for (int l = 7; l >= 0 && !below; --l) {
            if (x.v[l] > frc::MOD[l]) return false;
            below = x.v[l] < frc::MOD[l];
        }
        if (!below) return false;
        const Fr uk = fr_to_mont(x);
        for (size_t b = 0; b < size; ++b) {
            const Fr hi = fr_mul(out[b], uk);
            out[b + size] = hi;
            out[b] = fr_sub(out[b], hi);
        }
        size *= 2;
    }
    return true;
}

static bool host_fr_from_bytes(const zkdl_fr& a, Fr* mont) {
    Fr x;
    memcpy(x.v, a.le, 32);
    bool below = false;
    for (int l = 7; l >= 0 && !below; --l) {
        if (x.v[l] > frc::MOD[l]) return false;
        below = x.v[l] < frc::MOD[l];
    }
    if (!below) return false;
    *mont = fr_to_mont(x);
    return true;
}

extern "C" int hyrax_verify(zkdl_ctx* ctx, const zkdl_commit_key* key, const uint8_t* commitments, size_t nrows,
                            const zkdl_fr* point, size_t npoint, const zkdl_fr* T, const zkdl_fr* rho, const zkdl_fr* y,
                            int* verdict, uint8_t* combined_out) {
    if (!ctx || !key || !commitments || !T || !y || !verdict || (npoint && !point)) return ZKDL_EINVAL;
    if (nrows == 0 || (nrows & (nrows - 1)) || nrows > ((size_t)1 << 16)) return ZKDL_EINVAL;
    int lr = 0;
    while (((size_t)1 << lr) < nrows) ++lr;
    if ((int)npoint < lr || (int)npoint - lr > 15) return ZKDL_EINVAL;
    const int lc = (int)npoint - lr;
    const uint64_t cols = (uint64_t)1 << lc;
    if (cols > key->ncols) return ZKDL_EINVAL;
    *verdict = 1;
    // the weights of the rows and <T, beta~(v_col, .)> on the host (at most 2^16 + 2^15 products)
    std::vector<Fr> b_row, b_col;
    if (!host_beta_table(point, lr, b_row) || !host_beta_table(point + lr, lc, b_col)) return ZKDL_OK;
    Fr acc = fr_zero(), ym, rm = fr_zero();
    std::vector<uint32_t> scal(8 * (nrows + cols + 1) + 16, 0u);   // the last words: the kernels' error flag, zero
    for (uint64_t c = 0; c < cols; ++c) {
        Fr t;
        if (!host_fr_from_bytes(T[c], &t)) return ZKDL_OK;
        acc = fr_add(acc, fr_mul(b_col[c], t));
        uint32_t kw[8];
        memcpy(kw, T[c].le, 32);
        if (!glv_split(kw, &scal[8 * (nrows + c)])) return ZKDL_EINVAL;
    }
    if (!host_fr_from_bytes(*y, &ym) || (rho && !host_fr_from_bytes(*rho, &rm))) return ZKDL_OK;
    for (size_t j = 0; j < nrows; ++j) {
        const Fr plain = fr_from_mont(b_row[j]);
        if (!glv_split(plain.v, &scal[8 * j])) return ZKDL_EINVAL;
    }
    if (rho) {
        uint32_t kw[8];
        memcpy(kw, rho->le, 32);
        if (!glv_split(kw, &scal[8 * (nrows + cols)])) return ZKDL_EINVAL;
    }
    Fq beta;
    if (!endo_beta(&beta)) return ZKDL_EINVAL;
    ZK_HIP(ctx, hipSetDevice(ctx->device));
    // sum 1: the row commitments with the weights beta~(v_row, .); sum 2: Commit(T; rho*) on the key's generators
    const uint64_t n2 = cols + 1;
    const unsigned g1 = (unsigned)((nrows + MSM_TERMS - 1) / MSM_TERMS), g2 = (unsigned)((n2 + MSM_TERMS - 1) / MSM_TERMS);
    uint8_t* d_comm = (uint8_t*)zk_alloc(ctx, nrows * 96);
    uint32_t* d_scal = (uint32_t*)zk_alloc(ctx, scal.size() * 4);
    G1* d_part = (G1*)zk_alloc(ctx, sizeof(G1) * (g1 + g2));   // the blocks that check the subgroup write none
    G1* d_gens = (G1*)zk_alloc(ctx, sizeof(G1) * n2);   // G_0 .. G_{cols-1}, H
    uint8_t* d_out = (uint8_t*)zk_alloc(ctx, 256 + 2 * sizeof(G1));   // 2 x 96 bytes | the error flag's copy | 2 projective sums
    G1* d_proj = d_out ? (G1*)(d_out + 256) : nullptr;
    const bool affine = combined_out != nullptr;   // the bytes of C* are wanted: one inversion per sum
    int rc = (d_comm && d_scal && d_part && d_gens && d_out) ? ZKDL_OK : ZKDL_ENOMEM;
    uint8_t h_out[256];
    G1 h_proj[2];
    hipError_t e = hipSuccess;
    if (rc == ZKDL_OK) {
        e = hipMemcpyAsync(d_comm, commitments, nrows * 96, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = hipMemcpyAsync(d_scal, scal.data(), scal.size() * 4, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess)
            e = hipMemcpyAsync(d_gens, key->gens, sizeof(G1) * cols, hipMemcpyDeviceToDevice, ctx->stream);
        if (e == hipSuccess)
            e = hipMemcpyAsync(d_gens + cols, key->gens + key->ncols, sizeof(G1), hipMemcpyDeviceToDevice, ctx->stream);
        if (e == hipSuccess) {
            hipLaunchKernelGGL(k_msm_terms, dim3(g1 + g2 + g1), dim3(64), 0, ctx->stream, d_comm, (uint64_t)nrows, g1, d_gens,
                               n2, g2, d_scal, d_part, d_scal + 8 * (nrows + cols + 1), beta);
            hipLaunchKernelGGL(k_msm_finish, dim3(2), dim3(64), 0, ctx->stream, d_part, (uint64_t)g1, (uint64_t)g2, d_out,
                               affine ? (G1*)nullptr : d_proj);
            e = affine ? hipMemcpyAsync(h_out, d_out, 192, hipMemcpyDeviceToHost, ctx->stream)
                       : hipMemcpyAsync(h_proj, d_proj, 2 * sizeof(G1), hipMemcpyDeviceToHost, ctx->stream);
            if (e == hipSuccess)
                e = hipMemcpyAsync(h_out + 192, d_scal + 8 * (nrows + cols + 1), 4, hipMemcpyDeviceToHost, ctx->stream);
        }
    }
    hipError_t e2 = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess) e = e2;
    if (e == hipSuccess) e = hipGetLastError();
    zk_free(ctx, d_comm);
    zk_free(ctx, d_scal);
    zk_free(ctx, d_part);
    zk_free(ctx, d_gens);
    zk_free(ctx, d_out);
    if (rc != ZKDL_OK) return rc;
    ZK_HIP(ctx, e);
    uint32_t bad;
    memcpy(&bad, h_out + 192, 4);
    if (bad) return ZKDL_OK;                       // verdict 1: a commitment is not an element of the group
    if (combined_out) memcpy(combined_out, h_out, 96);
    bool same;
    if (affine) {
        same = memcmp(h_out, h_out + 96, 96) == 0;
    } else {   // X1 Z2 = X2 Z1 and Y1 Z2 = Y2 Z1 (the identity is (0, 1, 0): it equals only itself)
        const G1 &a = h_proj[0], &b = h_proj[1];
        same = fq_eq(fq_mul(a.X, b.Z), fq_mul(b.X, a.Z)) && fq_eq(fq_mul(a.Y, b.Z), fq_mul(b.Y, a.Z)) &&
               fq_is_zero(a.Z) == fq_is_zero(b.Z);
    }
    if (!same) {
        *verdict = 2;                              // Commit(T; rho*) is not the combined commitment
        return ZKDL_OK;
    }
    *verdict = fr_eq(acc, ym) ? 0 : 3;             // 3: <T, beta~(v_col, .)> != y
    return ZKDL_OK;
}
