// Internal declarations shared by the translation units of the library.
#pragma once
#include <stdint.h>
#include <stddef.h>
#include <map>
#include <vector>
#include <hip/hip_runtime.h>

#include "fr.cuh"
#include "sha256.cuh"
#include "../../include/zkdl.h"

constexpr int ZK_MAX_CHAL = 1024;          // challenges one call may draw
constexpr int ZK_PROOF_CAP = 1 << 17;      // proof bytes one call may write
constexpr int ZK_MAX_PART_BLOCKS = 1024;   // partial-sum slots of a round kernel
constexpr int ZK_MAX_EVALS = 4;            // evaluations per round polynomial (degree <= 3)
constexpr int ZK_BLOCK = 256;
constexpr int ZK_PEND_CAP = 448;         // bytes of host-known transcript frames waiting for the next transcript kernel
constexpr int ZK_STATE_HEAD = 128;       // bytes at the start of DevState that a call sets from the host

// Device-resident state of the call in flight.
struct DevState {
    uint32_t ts_state[8];   // transcript: SHA-256 chaining value after the last block of the stream
    uint32_t err;           // bit 0: zkReLU input out of range
    uint32_t ts_nblk[2];    // transcript: number of 64-byte blocks in the stream (low, high word)
    uint32_t lag_npts;      // != 0: claim is owed, claim = g(chal[lag_chal]) with the coefficients lag[]
    uint32_t lag_chal;
    uint32_t ts_fill;       // transcript: bytes of the unfinished block
    uint32_t pad0[2];
    uint32_t ts_buf[16];    // transcript: the unfinished block, big-endian words, zero beyond ts_fill
    Fr claim;               // claim of the running sumcheck (Montgomery); current if lag_npts == 0
    Fr lag[4];              // Lagrange coefficients of the last round polynomial
    Fr inv2, inv6;          // constants of the Lagrange formulas
    Fr weights[8];          // zkReLU: r^2, r, r'r^2, r'r, r'
    Fr scal[64];            // scalars handed between kernels (claims, finals)
    Fr chal[ZK_MAX_CHAL];   // challenges, Montgomery form
    uint8_t chal_le[ZK_MAX_CHAL * 32];
    uint8_t proof[ZK_PROOF_CAP];
};

enum TensorKind { TK_FR = 0, TK_I32 = 1, TK_I64 = 2 };

struct zkdl_tensor {
    int kind;
    int ndim;
    uint64_t shape[ZKDL_MAX_DIMS];
    uint64_t numel;
    void* data;      // TK_FR: uint32_t planes (8 * numel words); else the integers
    bool owned;
};

struct zkdl_transcript {
    ts::State s;
};

constexpr int ZK_MAX_PATCHES = 64;       // proof-header records of one call
struct HeaderPatch {
    size_t off;
    uint32_t words[8];
    int n;
};

struct zkdl_ctx {
    int device;
    hipStream_t stream;
    int last_hip;
    DevState* dev;            // device
    uint8_t* host_stage;      // pinned host staging (sizeof(DevState))
    Fr* partials;             // device: ZK_MAX_PART_BLOCKS * ZK_MAX_EVALS * 2 partial sums
    void* static_scratch;     // device address, on this context's device, of the library's static work memory
    std::multimap<size_t, void*> free_blocks;
    std::map<void*, size_t> live_blocks;
    // per-call bookkeeping (host mirrors of device cursors)
    int n_chal;
    size_t proof_len;
    HeaderPatch patches[ZK_MAX_PATCHES];
    int n_patches;
    bool patch_overflow;
    // transcript frames known on the host (protocol headers) that the next transcript
    // kernel absorbs before anything else
    uint8_t pend[ZK_PEND_CAP];
    uint32_t pend_len;
    // zkReLU: the columns of a round are cut into chunks until this many threads are busy
    uint64_t zk_fill_threads;
    // commitment keys: bits per window of a tensor entry's table (0: chosen by table size; 8 or 12)
    int commit_wbits;
    // optional per-kernel-class timing with HIP events on the context's stream
    bool prof_on;
    struct ProfSpan {
        hipEvent_t e0, e1;
        int cls;
    };
    std::vector<ProfSpan> prof_spans;   // pool; the first prof_used are pending
    size_t prof_used;
    double prof_ms[ZKDL_PROF_CLASSES];
    double prof_bytes[ZKDL_PROF_CLASSES];
    uint64_t prof_launches[ZKDL_PROF_CLASSES];
};

// Brackets one kernel launch when profiling is on; `bytes` = algorithmic bytes it moves.
void zk_prof_begin(zkdl_ctx* ctx, int cls, double bytes);
void zk_prof_end(zkdl_ctx* ctx);

#define ZK_HIP(ctx, call)                       \
    do {                                        \
        hipError_t e__ = (call);                \
        if (e__ != hipSuccess) {                \
            (ctx)->last_hip = (int)e__;         \
            return ZKDL_EHIP;                   \
        }                                       \
    } while (0)

// scratch allocator of the context (caches freed blocks)
void* zk_alloc(zkdl_ctx* ctx, size_t bytes);
void zk_free(zkdl_ctx* ctx, void* p);

static inline FrTab make_tab(void* p, uint64_t ps) {
    FrTab t;
    t.p = (uint32_t*)p;
    t.ps = ps;
    return t;
}
static inline FrTab tab_offset(const FrTab& t, uint64_t elems) {
    FrTab o = t;
    o.p += elems;
    return o;
}

// ---- k_basic.hip -------------------------------------------------------------
void zk_launch_convert(zkdl_ctx* ctx, const void* src, int kind_or_le, uint64_t n, FrTab out);
void zk_launch_download(zkdl_ctx* ctx, FrTab in, uint64_t n, uint8_t* out_le_dev);
void zk_launch_points_to_mont(zkdl_ctx* ctx, const uint8_t* le_dev, int n, Fr* out);
// chal[dst .. dst + n) = given coordinates: canonical little-endian bytes on the device, or
// (le_dev == nullptr) copies of chal[idx->v[i]]; n <= ZK_CHAL_SET_MAX
constexpr int ZK_CHAL_SET_MAX = 128;
struct ChalIdx {
    int16_t v[ZK_CHAL_SET_MAX];
};
void zk_launch_chal_set(zkdl_ctx* ctx, int dst, int n, const uint8_t* le_dev, const ChalIdx* idx);
// beta~(point, .) for the m challenges point[0..m) (device, Montgomery, AoS)
int zk_build_beta(zkdl_ctx* ctx, const Fr* point, int m, FrTab out);
// several tables with two launches in all (tables of more than 2^22 entries are built one by one)
struct BetaJob {
    const Fr* point;   // device, Montgomery form, m coordinates
    int m;
    FrTab out;         // 2^m entries
};
int zk_build_beta_many(zkdl_ctx* ctx, const BetaJob* jobs, int n);
// out[o, i] = sum_a beta[a] * src[o, a, i]; src kind TK_*; out has O * I elements
int zk_partial_eval(zkdl_ctx* ctx, int kind, const void* src, uint64_t O, uint64_t A, uint64_t I,
                    FrTab beta, FrTab out);
void zk_launch_broadcast_rows(zkdl_ctx* ctx, FrTab src, uint64_t rows, uint64_t inner, FrTab out);
void zk_launch_soa_to_aos(zkdl_ctx* ctx, FrTab in, int n, Fr* out);
void zk_launch_shift_rows(zkdl_ctx* ctx, FrTab src, uint64_t rows, uint64_t inner, uint32_t period,
                          FrTab out);

// ---- k_sumcheck.hip ------------------------------------------------------------
// Runs all rounds of a degree-K product sumcheck on K packed tables of length 2^d.
// The sources are read only; work_mem (zk_sumcheck_work_bytes(K, d) bytes) receives the
// folded tables.  Writes one SC block at ctx->proof_len, draws d challenges.
size_t zk_sumcheck_work_bytes(int K, int d);
int zk_sumcheck_product(zkdl_ctx* ctx, int K, const FrTab* src, void* work_mem, int d,
                        int finals_scal_base);
// The product sumcheck on (beta~(p, .), X0, X1) for 2^d entries, d >= ZK_HD_MIN_LOG, with two folded
// tables: the same proof bytes and transcript as zk_sumcheck_product on the three tables.  x: X0, X1
// packed; wsuf[t], t < d - 10: beta~(p_[t+1:], .), 2^(d-t-1) entries; eq_tail: 2^11 work-table
// entries of scratch; work_mem: zk_sumcheck_work_bytes(2, d); p_idx: challenge index of p_0.
constexpr int ZK_HD_MIN_LOG = 14;
// wsuf[t_last] built; fills wsuf[t_last - 1] .. wsuf[t_first], each from the one after it
void zk_hadamard_suffix_tables(zkdl_ctx* ctx, const FrTab* wsuf, int t_last, int t_first, int d, int p_idx);
// xi != nullptr: X0, X1 are int32 arrays on the device; the first two rounds read them, x and wsuf[0] are
// unused and the first round's weights are split[0][b >> split_lb] * split[1][b & (2^split_lb - 1)]
// (beta~ of the leading d - 1 - split_lb and of the last split_lb coordinates of p_[1:]).
int zk_hadamard_eq(zkdl_ctx* ctx, const FrTab* x, const int32_t* const* xi, const FrTab* wsuf, const FrTab* split,
                   int split_lb, void* work_mem, F9Tab eq_tail, int d, int p_idx, int finals_scal_base);
// Queues the frame of a protocol header (label, n <= 8 little-endian u32 words); it is absorbed
// by the next zk_launch_draw / zk_flush_frames, in stream order before everything that follows.
void zk_absorb_words(zkdl_ctx* ctx, const char* label, const uint32_t* words, int n);
// absorbs the queued frames, then draws `count` challenges into chal[chal_base ..)
void zk_launch_draw(zkdl_ctx* ctx, int chal_base, int count);
static inline void zk_flush_frames(zkdl_ctx* ctx) { zk_launch_draw(ctx, 0, 0); }

// ---- k_reindex.hip ---------------------------------------------------------------
struct ReindexJob {
    int K;
    const int32_t* map[ZKDL_REINDEX_MAX_K];   // device: stack index of the j-th tensor of sub-stack k, -1 = zero
    uint64_t len[ZKDL_REINDEX_MAX_K];
    FrTab beta[ZKDL_REINDEX_MAX_K];           // beta~(u_k, .)
    const uint32_t* row_off;                  // device: inverse maps by stack index, 2^ln + 1 offsets into ent
    const uint32_t* ent;                      // device: k in the top 3 bits, j in the other 29
};
// claims of the sub-stacks -> scal[8 ..), absorbed and written to the proof; K coefficients drawn;
// P built into p; product sumcheck on (p, t) over ln variables, finals at scal[0], scal[1]
int zk_reindex(zkdl_ctx* ctx, const ReindexJob& job, FrTab t, FrTab p, int ln, void* work_mem);
// maps of a chained window built on the device: maps [K N], row_off [N + 1], ent [K N], K = 1 + with_ident
void zk_launch_layer_maps(zkdl_ctx* ctx, uint32_t N, uint32_t L, int with_ident, int32_t* maps, uint32_t* row_off,
                          uint32_t* ent);

// claims st->scal[scal_base .. + K) absorbed under "c" and written to the proof at proof_off, then n_draw challenges
// drawn into chal[chal_base ..)
void zk_launch_absorb_claims(zkdl_ctx* ctx, int scal_base, int K, uint32_t proof_off, int chal_base, int n_draw);

// K claims X~(p_k) on the table x (2^d entries) -> one: the claims -> scal[8 ..), absorbed and written
// to the proof; K coefficients drawn; P = sum_k r_k beta[k] built into p; product sumcheck on (p, x),
// finals at scal[0], scal[1]
int zk_merge(zkdl_ctx* ctx, int K, const FrTab* beta, FrTab x, FrTab p, int d, void* work_mem);

// The same for a stack X [N, rows * cols] on tables of the inner size: claim k at the ln + ld
// challenges from point[k] on (stack coordinates first).  Claims -> scal[8 ..) and the proof; K
// coefficients drawn; two product sumchecks (inner over (k, x), then over the stack index), the last
// finals at scal[0], scal[1].  The work memory is appended to `keep` (free it once the stream has
// drained).
struct StackMergeJob {
    int K;
    const Fr* point[ZKDL_REINDEX_MAX_K];   // device, Montgomery form
    int kind;                              // TK_*
    const void* X;                         // TK_FR: const FrTab*; else the integers (device)
    uint64_t N, rows, cols;
};
int zk_stack_merge(zkdl_ctx* ctx, const StackMergeJob& job, std::vector<void*>& keep);

// ---- k_zkrelu.hip ----------------------------------------------------------------
// optimized aggregated matrix-product protocol: stack rounds with f_t, then the single-product sumcheck
int zk_matmul_ft(zkdl_ctx* ctx, const FrTab* src, void* work_mem, int ln, int l2, const FrTab* wsuf, int w_idx,
                 int finals_scal_base);
// given_points != 0: u_Z, u_A, u_GA, u_GZ already stand in chal[n_chal .. n_chal + 4 log2 D); only u_bin is drawn
int zk_zkrelu(zkdl_ctx* ctx, const int64_t* z_dev, const int64_t* ga_dev, uint64_t D, int Q, int R,
              int given_points);

// ---- k_general.hip -----------------------------------------------------------------
// the batched matrix product in the general aggregated form: header frame, draw of (w, u), the "ZKGA"
// block; finals Y~, X0~, X1~ -> scal[scal_base ..), scal[scal_base + 3] is used as well
int zk_matmul_general(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1, const zkdl_tensor* Y, int ln,
                      int l1, int l2, int l3, int scal_base);

// ---- api.hip -----------------------------------------------------------------------
size_t zk_claims_unlinked(zkdl_claim* claims_out, const uint8_t* proof, uint32_t L, uint32_t B, uint32_t width, uint32_t T,
                          uint32_t Q, uint32_t R, int cf, size_t pf, int ca, size_t pa, int cw, size_t pw, int cz, size_t pz,
                          size_t pend);
void zk_write_proof_words(zkdl_ctx* ctx, const uint32_t* words, int n);   // appends a header
void zk_host_absorb_u32(zkdl_transcript* t, const char* label, const uint32_t* words, int n);
