/* zkdl.h - C ABI of the MI355X tensor-sumcheck prover for zkDL (arXiv 2307.16273).
 *
 * The library proves, on one gfx950 GPU, the sumcheck instances that zkDL uses
 * for a training step over the BLS12-381 scalar field Fr: multilinear-extension
 * partial evaluations (Sec. 2.2, Eq. multilinear-extension), batched matrix and
 * Hadamard products (Sec. 4, Eqs. exm-matmul-batched, exm-hadamard-batched),
 * zkReLU (Sec. 3.1, App. A) and their aggregation over layers and steps (Sec. 5,
 * Protocol zkdl, the sumcheck line).  The verifier's random messages of the
 * interactive protocols (App. B) are replaced by a SHA-256 Fiat-Shamir
 * transcript that runs on the device next to the kernels.
 *
 * Conventions
 *  - Every function returns ZKDL_OK (0) or a negative zkdl_err; nothing aborts
 *    or throws.  After ZKDL_EHIP, zkdl_last_hip_error() gives the HIP code.
 *  - "host" / "device" is stated for every pointer.  The caller owns every
 *    buffer it passes; the library owns zkdl_tensor storage and its scratch.
 *  - Field elements cross the boundary as zkdl_fr: 32 bytes, canonical (fully
 *    reduced), little-endian, NOT in Montgomery form.
 *  - Tensors are row-major, every dimension a power of two (pad with zeros
 *    otherwise, Sec. 2.2).  A point is the concatenation of one vector per
 *    axis, leading axis first; inside an axis coordinate 0 pairs with the most
 *    significant bit of that axis' index.
 *  - A call enqueues its kernels on the context's stream and returns after the
 *    proof bytes have been copied to the caller's host buffer (it synchronises
 *    that stream once, at the end).  Calls on one context must not overlap.
 *  - points_out / npoints: if points_out != NULL, *npoints holds its capacity
 *    on entry; on return the challenges drawn during the call are stored in
 *    draw order and *npoints is their number (ZKDL_ESMALL if too small).
 *  - proof / proof_len: *proof_len holds the capacity in bytes on entry and the
 *    bytes written on return.  If the proof or the points buffer is too small
 *    the call returns ZKDL_ESMALL with *proof_len and *npoints set to the sizes
 *    needed and nothing else of the caller's changed: the transcript stays where
 *    it was, so the same call with larger buffers gives the proof a verifier
 *    replays.  proof == NULL with proof_len != NULL is that size query;
 *    proof_len == NULL means the caller does not want the bytes.
 *
 * Transcript (this library's own format).  The transcript is one byte stream;
 * every value derived from it is a plain SHA-256 of an extension of it:
 *   stream_0         = "zkdl-mi355x/v3" zero-padded to 56 bytes || u64le(seed)
 *   absorb(label, m) : stream <- stream || u8(|label|) || label || u64le(|m|)
 *                      || m, |label| <= 32
 *   challenges(n)    : c_i = int_le(SHA256(stream || 0xF0 || u32le(i)) ||
 *                      SHA256(stream || 0xF1 || u32le(i))) mod r for i < n,
 *                      then stream <- stream || 0xF2 || zero bytes up to the
 *                      next multiple of 64
 *   digest           = SHA256(stream)
 * Field elements are absorbed as zkdl_fr bytes.  A sumcheck absorbs its header
 * words under the protocol's name, claim_0 under "c" (where the verifier cannot
 * compute it), per round g_t(0), g_t(2), .., g_t(degree) under "g" (g_t(1) is
 * fixed by the round check g_t(0) + g_t(1) = claim, Sec. 2.2) followed by a
 * draw of one challenge, and the finals under "f".
 *
 * Proof layout (all integers little-endian u32, all field elements zkdl_fr)
 *   SC block : "ZKSC", n_finals, degree, rounds, claim_0,
 *              rounds x (degree+1) evaluations g_t(0..degree), n_finals finals
 *   zkReLU   : "ZKRL", log2 D, Q, R, has_ga, mode, 0, 0 (mode 0: all points drawn;
 *              1, 2: the four points given, see zkrelu_prove_at), four input claims
 *              (Z, A, G_A, G_Z), SC block (degree 3, finals aux~(0,v,w),
 *              aux~(1,v,w), aux~(0,v,Q+R-1)), SC block of the merge (degree 2,
 *              finals aux~(k*,v,w*), E~(k*,w*))
 *   aggregate: "ZKAG", L, B, width, T', Q, R, 0, SC block forward, SC block
 *              gradA, SC block gradW, zkReLU proof
 *   "ZKUP" (update_prove), "ZKGA" (sumcheck_matmul_general), "ZKSF" (sumcheck_matmul_ft), "ZKRI" (reindex_prove), "ZKMG"
 *   (claims_merge_prove), "ZKMS" (claims_merge_stack_prove) and "ZKAL"
 *   (aggregate_prove_linked) are laid out at their declarations below.
 * points_out also repeats, in front of the draws they precede, points that a
 * call hands on from earlier challenges (aggregate_prove_linked).
 */
#ifndef ZKDL_H
#define ZKDL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZKDL_OK = 0,
    ZKDL_EINVAL = -1, /* null pointer, bad dtype, dimension not a power of two, shape mismatch */
    ZKDL_ERANGE = -2, /* a zkReLU input is not a (Q+R)-bit signed integer (Theorem completeness) */
    ZKDL_ENOMEM = -3, /* device or host allocation failed */
    ZKDL_EHIP = -4,   /* a HIP runtime call failed */
    ZKDL_ESMALL = -5, /* an output buffer is too small */
    ZKDL_ETOOBIG = -6 /* the input exceeds the fixed work memory of an allocation-free entry point */
} zkdl_err;

typedef enum { ZKDL_I32 = 0, ZKDL_I64 = 1, ZKDL_FR_LE = 2 } zkdl_dtype;

typedef struct zkdl_ctx zkdl_ctx;               /* device id + borrowed hipStream_t + scratch */
typedef struct zkdl_tensor zkdl_tensor;         /* device tensor: Fr (SoA limb planes, Montgomery) or borrowed integers */
typedef struct zkdl_transcript zkdl_transcript; /* SHA-256 Fiat-Shamir state, host side */
typedef struct { uint8_t le[32]; } zkdl_fr;

#define ZKDL_MAX_DIMS 4

/* ---- context ------------------------------------------------------------ */
/* hip_stream: a hipStream_t (e.g. torch.cuda.current_stream().cuda_stream), or
 * NULL for the default stream.  The stream is borrowed, never destroyed. */
int zkdl_ctx_create(zkdl_ctx** out, int device, void* hip_stream);
int zkdl_ctx_destroy(zkdl_ctx* ctx);
int zkdl_last_hip_error(const zkdl_ctx* ctx);
/* Tuning: zkrelu_prove cuts the bit columns of a round into chunks (more threads per row pair)
 * until about `threads` threads are busy; the default, 65536, is one wave on every SIMD of the
 * device.  The same figure decides from which size on the later rounds of its linear equations keep the
 * equality tables as two factors and round 4 of the binarity sum runs on the integers.  Proofs do not
 * depend on it.  1 <= threads <= 2^24, else ZKDL_EINVAL. */
int zkdl_ctx_set_fill_threads(zkdl_ctx* ctx, uint64_t threads);
/* Tuning: bits per window of the fixed-base tables that zkdl_commit_key_create builds for tensor entries from
 * now on: 8, 12, or 0 (the default) for 12 while a key's tables stay below 16 GiB and 8 otherwise.  Commitments
 * do not depend on it.  Another value: ZKDL_EINVAL. */
int zkdl_ctx_set_commit_window_bits(zkdl_ctx* ctx, int bits);
const char* zkdl_strerror(int err);
/* Frees cached scratch memory (the context keeps freed blocks for reuse). */
int zkdl_ctx_trim(zkdl_ctx* ctx);

/* ---- transcript (host side; format in the header comment of this file) ---
 * absorb: label is a NUL-terminated string of at most 32 bytes (ZKDL_EINVAL
 * otherwise); host_bytes may be NULL when n is 0.  challenge: one draw of one
 * element.  digest: SHA-256 of the stream so far; does not change the state. */
int zkdl_transcript_create(zkdl_transcript** out, uint64_t seed);
int zkdl_transcript_destroy(zkdl_transcript* t);
int zkdl_transcript_absorb(zkdl_transcript* t, const char* label, const void* host_bytes, size_t n);
int zkdl_transcript_challenge(zkdl_transcript* t, zkdl_fr* host_out);
int zkdl_transcript_digest(const zkdl_transcript* t, uint8_t host_out[32]);

/* ---- tensors --------------------------------------------------------------
 * fr_tensor_upload: the discretised tensor of Sec. 2.2 mapped into Fr.  src is
 * `numel` items of dtype (ZKDL_I32 / ZKDL_I64: signed, x -> x mod r;
 * ZKDL_FR_LE: 32-byte little-endian values, reduced mod r), in host memory or,
 * if src_on_device != 0, in device memory.  The result is Fr in Montgomery
 * form, eight 32-bit limb planes (structure of arrays). */
int fr_tensor_upload(zkdl_ctx* ctx, const void* src, int dtype, int src_on_device,
                     const uint64_t* shape, int ndim, zkdl_tensor** out);
/* A view of integers already in device memory (no copy, memory stays the
 * caller's and must outlive the tensor).  Accepted wherever a tensor is read;
 * the conversion into Fr happens inside the consuming kernel. */
int zkdl_tensor_wrap_int(zkdl_ctx* ctx, const void* device_src, int dtype, const uint64_t* shape,
                         int ndim, zkdl_tensor** out);
int zkdl_tensor_ndim(const zkdl_tensor* t);
uint64_t zkdl_tensor_dim(const zkdl_tensor* t, int axis);
uint64_t zkdl_tensor_numel(const zkdl_tensor* t);
/* Canonical bytes of every element, row-major, into host memory (numel x 32 B). */
int zkdl_tensor_download(zkdl_ctx* ctx, const zkdl_tensor* t, zkdl_fr* host_out);
int zkdl_tensor_free(zkdl_ctx* ctx, zkdl_tensor* t);

/* ---- MLE partial evaluation (Eq. multilinear-extension, Sec. 2.2) ----------
 * Binds the variables of axes [axis_lo, axis_hi) to `point` (host, npoint =
 * sum of log2 of those dimensions):
 *   out[o, i] = sum_a beta~(point, a) * t[o, a, i].
 * The result has the remaining axes (ndim 0 = a single element). */
int mle_partial_eval(zkdl_ctx* ctx, const zkdl_tensor* t, int axis_lo, int axis_hi,
                     const zkdl_fr* point, size_t npoint, zkdl_tensor** out);

/* ---- sumchecks -------------------------------------------------------------
 * sumcheck_product: sum over the hypercube of the product of K (1..3) Fr
 * tensors of equal numel 2^d, degree-K round polynomials (Sec. 2.2).  The
 * inputs are not modified.  finals (host, K elements, may be NULL): the tables'
 * evaluations at the challenge point.  Transcript: header "sumcheck_product"
 * (K, d), claim_0, the rounds, the finals.  Proof: one SC block. */
int sumcheck_product(zkdl_ctx* ctx, const zkdl_tensor* const* tables, int K, zkdl_transcript* tr,
                     uint8_t* proof, size_t* proof_len, zkdl_fr* finals, zkdl_fr* points_out,
                     size_t* npoints);

/* sumcheck_product_noalloc: sumcheck_product for callers that cannot allocate device memory while
 * they run - code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, transcript, proof bytes and results as sumcheck_product.  The folded tables live
 * in a static device array of the library (3 x 2^(ZKDL_NOALLOC_MAX_LOG2 - 1) x 36 bytes = 13.5 MiB,
 * held by every GPU the library runs on until the process ends) whose address on the context's
 * device is taken when the context is created; the call itself makes no hipMalloc / hipFree and no
 * other allocation, on the device or the host.  Limits: every table an Fr tensor (an integer view
 * would need a converted copy: ZKDL_EINVAL), at most 2^ZKDL_NOALLOC_MAX_LOG2 entries per table
 * (ZKDL_ETOOBIG beyond, nothing is enqueued and the transcript is untouched), per-kernel timing
 * switched off (ZKDL_EINVAL).  All calls on one GPU share the one array: calls that overlap on a GPU,
 * from different contexts or streams, race; calls on one context follow each other on its stream and
 * need nothing cleared in between. */
#define ZKDL_NOALLOC_MAX_LOG2 18
int sumcheck_product_noalloc(zkdl_ctx* ctx, const zkdl_tensor* const* tables, int K, zkdl_transcript* tr,
                             uint8_t* proof, size_t* proof_len, zkdl_fr* finals, zkdl_fr* points_out,
                             size_t* npoints);

/* sumcheck_matmul: Eq. exm-matmul-batched,
 *   Y~(w,u0,u1) = sum_n sum_i beta~(w,n) X0~(n,u0,i) X1~(n,i,u1)
 * for Y[n] = op(X0[n]) op(X1[n]).  X0, X1 are 3-d tensors with the stack axis
 * first; transpose_xk != 0 means op() transposes the stored matrices (the
 * kernel binds the other axis; nothing is copied).  Logical shapes
 * op(X0[n]) [D1,D2], op(X1[n]) [D2,D3].  Draws w (log N), u0 (log D1),
 * u1 (log D3), then one challenge per round (n variables first, then i).
 * claims (host, 3 elements, may be NULL): Y~(w,u0,u1), X0~(v_n,u0,v_i),
 * X1~(v_n,v_i,u1).  Proof: one SC block with K = 3 (beta~(w,.) is a table). */
int sumcheck_matmul(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1, int transpose_x0,
                    int transpose_x1, zkdl_transcript* tr, uint8_t* proof, size_t* proof_len,
                    zkdl_fr* claims, zkdl_fr* points_out, size_t* npoints);

/* sumcheck_matmul_ft: the same statement with the prover's messages of the optimized
 * aggregated protocol (App. B, Protocol tensor-op-aggr-optimized).  For the log N stack
 * rounds the prover sends f_t(0), f_t(1), f_t(2), the round polynomial without its
 * factor beta~(w_t, .), which the verifier multiplies back:
 *   f_t(x) = sum_{n'} beta~(w_[t+1:], n') sum_i X0~(v_<t, x, n', u0, i) X1~(v_<t, x, n', i, u1),
 *   (1 - w_t) f_t(0) + w_t f_t(1) = claim,  next claim f_t(v_t);
 * beta~(w, .) is never folded and the messages have degree 2.  Then the sumcheck of the
 * single product sum_i X0~(v_n, u0, i) X1~(v_n, i, u1) follows (Eq.
 * tensor-op-compressed-optimized): K = 2, degree 2.  Arguments and claims as for
 * sumcheck_matmul.  Transcript: header "sumcheck_matmul_ft" (N, D1, D2, D3), one draw
 * (w, u0, u1), "c" claim_0, per stack round "f" (three evaluations) and a draw, then the
 * product sumcheck's rounds and finals (its claim_0 is not absorbed again).
 * Proof: "ZKSF", log2 N, log2 D2, 0, claim_0, log2 N x 3 evaluations, then one SC block
 * (K = 2, claim_0 = f_{n-1}(v_{n-1}), finals X0~(v_n,u0,v_i), X1~(v_n,v_i,u1)). */
int sumcheck_matmul_ft(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1, int transpose_x0,
                       int transpose_x1, zkdl_transcript* tr, uint8_t* proof, size_t* proof_len,
                       zkdl_fr* claims, zkdl_fr* points_out, size_t* npoints);

/* sumcheck_matmul_general: N products Y[n] = X0[n] X1[n] proved from the three stacks
 * themselves, in the general aggregated form (Sec. 4, Eq. tensor-op-aggr with f(a, b) = a b;
 * Protocol tensor-op-aggr):
 *   0 = sum_n sum_i sum_j beta~(w,n) beta~(u,i) (D2^-1 Y(n,i) - X0(n,i0,j) X1(n,j,i1)),
 * i = (i0, i1) the output index, j the inner index; w (log N) and u = (u0, u1) (log D1 + log D3)
 * are drawn.  log N stack rounds with f_t(0), f_t(1), f_t(2), the round polynomial without its
 * factor beta~(w_t, .): (1 - w_t) f_t(0) + w_t f_t(1) = claim (0 at first), next claim f_t(v_t).
 * Then the sumcheck of Eq. tensor-op-compressed over (i0, i1, j) in that order, degree 2, whose
 * claim_0 = f_{n-1}(v_{n-1}) (0 without stack rounds) the transcript already fixes.  The verifier
 * ends with beta~(u, v_i) (D2^-1 Y~ - X0~ X1~) = last claim.
 * X0 [N, D1, D2], X1 [N, D2, D3], Y [N, D1, D3], stored as given (no transposes), any kind;
 * D1, D2, D3 <= 2^16 (ZKDL_ETOOBIG), N <= 2^13.  A Y that is not the product gives a proof the
 * verifier rejects: the prover does not check it.
 * claims (host, 3, may be NULL): Y~(v_n, v_i0, v_i1), X0~(v_n, v_i0, v_j), X1~(v_n, v_j, v_i1).
 * points_out: w, u0, u1, v_n, v_i0, v_i1, v_j (2 log N + 2 log D1 + 2 log D3 + log D2 elements).
 * Transcript: header "tensor_op_aggr" (N, D1, D2, D3), one draw (w, u), per stack round "f"
 * (three evaluations) and a draw, then the rounds ("g") and the finals ("f") of the SC block.
 * Proof: "ZKGA", log2 N, log2 D1, log2 D3, log2 D2, 0, 0, 0; log2 N x 3 evaluations; one SC block
 * (3 finals, degree 2, log2 D1 + log2 D3 + log2 D2 rounds). */
int sumcheck_matmul_general(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1, const zkdl_tensor* Y,
                            zkdl_transcript* tr, uint8_t* proof, size_t* proof_len, zkdl_fr* claims,
                            zkdl_fr* points_out, size_t* npoints);

/* sumcheck_hadamard: Eq. exm-hadamard-batched over the whole stack,
 *   Y~(p) = sum_b beta~(p,b) X0(b) X1(b),  p drawn over all log2(numel) variables.
 * claims (host, 3, may be NULL): Y~(p), X0~(v), X1~(v). */
int sumcheck_hadamard(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1,
                      zkdl_transcript* tr, uint8_t* proof, size_t* proof_len, zkdl_fr* claims,
                      zkdl_fr* points_out, size_t* npoints);

/* reindex_prove: the re-indexing sumcheck (Sec. 4, Eq. sc-reindex; the re-indexing line of
 * Protocol zkdl).  X is a stack of N = dim 0 tensors of D = numel / N elements (any kind).
 * K (1..ZKDL_REINDEX_MAX_K) sub-stacks X_k take tensors of it in their own order:
 * maps[k] (host, map_len[k] entries, a power of two up to 2^29) holds the stack index of the
 * j-th tensor of X_k, or -1 for a zero tensor (padding); an index may occur more than once.
 * Each sub-stack comes with a claim X_k~(points[k], u): points[k] (host, log2 map_len[k]
 * elements) over its stack axis, u (host, log2 D elements) over the rest.  The call computes
 * those K claims, draws coefficients r_k, and proves
 *   sum_k r_k X_k~(points[k], u) = sum_i P[i] X~(i, u),
 *   P[i] = sum_k r_k sum_{j : maps[k][j] = i} beta~(points[k], j),
 * by a sumcheck over i on the tables P and X~(., u) (K = 2, degree 2), which leaves the one
 * claim X~(v, u) on the whole stack; P~(v) is for the verifier to recompute from the maps.
 * claims (host, K + 2 elements, may be NULL): the K sub-stack claims, P~(v), X~(v, u).
 * Transcript: "reindex" with the SHA-256 digest of the statement's public part
 *   u32le N, D, K; per k: u32le map_len[k], the entries as i32le; the points in order k,
 *   32 B little-endian per element; u;
 * "c" the K claims; one draw of K coefficients; then the product sumcheck (claim_0, rounds,
 * finals).  Proof: "ZKRI", N, D, K, the K claims, one SC block.
 * Errors: ZKDL_EINVAL for a map entry outside [-1, N), sizes that are no powers of two,
 * D above 2^31 or a points argument that is NULL where elements are needed. */
#define ZKDL_REINDEX_MAX_K 8
int reindex_prove(zkdl_ctx* ctx, const zkdl_tensor* X, int K, const int32_t* const* maps,
                  const uint64_t* map_len, const zkdl_fr* const* points, const zkdl_fr* u,
                  zkdl_transcript* tr, uint8_t* proof, size_t* proof_len, zkdl_fr* claims,
                  zkdl_fr* points_out, size_t* npoints);

/* claims_merge_prove: K <= 8 claims X~(p_k) on one tensor X (2^d entries, every p_k over all d
 * variables, most significant index bit first) become one claim X~(v).  With coefficients r_k
 * from the verifier,  sum_k r_k X~(p_k) = sum_b P[b] X(b),  P = sum_k r_k beta~(p_k, .), by the
 * definition of the multilinear extension (Sec. 2.2); it is Eq. sc-reindex with every sub-stack
 * the stack itself and the sum taken over all variables, and yields the single evaluation per
 * stack that Protocol zkdl opens.  A product sumcheck on (P, X) proves it; the verifier
 * computes P~(v) = sum_k r_k beta~(p_k, v).
 * points (host): K arrays of d canonical elements.  claims (host, K + 2, may be NULL): the K
 * claims, P~(v), X~(v).  Transcript: "merge" with the SHA-256 digest of u32le d, K and the
 * points' bytes; "c" the K claims; one draw of K coefficients; the product sumcheck (claim_0,
 * rounds, finals).  Proof: "ZKMG", d, K, 0, the K claims, one SC block.
 * Errors: ZKDL_EINVAL for a size that is no power of two or above 2^30, K out of range, a
 * NULL or non-canonical point. */
int claims_merge_prove(zkdl_ctx* ctx, const zkdl_tensor* X, int K, const zkdl_fr* const* points,
                       zkdl_transcript* tr, uint8_t* proof, size_t* proof_len, zkdl_fr* claims,
                       zkdl_fr* points_out, size_t* npoints);

/* claims_merge_stack_prove: the same statement for a stack X [N, ...] (D = numel / N) on tables
 * of D, not N D, entries.  Claim k is X~(s_k, q_k), its point = s_k over the stack axis followed
 * by q_k over the rest.  With T[k, x] = X~(s_k, x) and E[k, x] = r_k beta~(q_k, x) (k padded
 * with zero rows to a power of two),
 *   sum_k r_k X~(s_k, q_k) = sum_{k, x} E[k, x] T[k, x]:
 * a product sumcheck over (k, x), k leading, with challenges (rho, v), leaves
 * T~(rho, v) = sum_k beta~(rho, k) X~(s_k, v), claims with one common inner point, and Eq.
 * sc-reindex, T~(rho, v) = sum_i Pn[i] X~(i, v), Pn[i] = sum_k beta~(rho, k) beta~(s_k, i), a
 * product sumcheck over i, leaves X~(v_n, v).  The verifier computes E~(rho, v), Pn~(v_n) and
 * checks that the second sumcheck starts from the first one's final on T.
 * claims (host, K + 2, may be NULL): the K claims, Pn~(v_n), X~(v_n, v).
 * Transcript: "merge_stack" with the SHA-256 digest of u32le N, D, K and the points' bytes;
 * "c" the K claims; one draw of K; the two product sumchecks, each with its claim_0.
 * Proof: "ZKMS", N, D, K, the K claims, two SC blocks.  Errors as claims_merge_prove. */
int claims_merge_stack_prove(zkdl_ctx* ctx, const zkdl_tensor* X, int K, const zkdl_fr* const* points,
                             zkdl_transcript* tr, uint8_t* proof, size_t* proof_len, zkdl_fr* claims,
                             zkdl_fr* points_out, size_t* npoints);

/* zkrelu_prove: the combined sumcheck of App. A over aux in {0,1}^{2 x D x (Q+R)}
 * (bit axis padded to a power of two), weights r^2, r, 1, r'r^2, r'r, r', then the
 * merge of the three claims on aux into one.  Z, GA: D signed (Q+R)-bit
 * integers each (host, or device if src_on_device != 0); GA == NULL is the
 * forward-only use and stands for G_A = 0.  D a power of two, Q + R <= 64,
 * R >= 1.  ZKDL_ERANGE if a value is out of range (the proof is then not
 * produced).  claims (host, 4, may be NULL): Z~(u_Z), A~(u_A), G_A~(u_GA),
 * G_Z~(u_GZ).  Draw order: u_Z, u_A, u_GA, u_GZ, u_bin, r, r', rounds, rho0..2,
 * merge rounds. */
int zkrelu_prove(zkdl_ctx* ctx, const int64_t* Z, const int64_t* GA, uint64_t D, int Q, int R,
                 int src_on_device, zkdl_transcript* tr, uint8_t* proof, size_t* proof_len,
                 zkdl_fr* claims, zkdl_fr* points_out, size_t* npoints);

/* zkrelu_prove_at: the same proof with the four points of the input claims given by the
 * caller instead of drawn (Sec. 3.2, App. A: they are the points that the sumchecks of the
 * operations Z, A, G_A, G_Z take part in have left).  points (host): 4 log2 D canonical
 * elements, u_Z, u_A, u_GA, u_GZ in this order, each with the most significant index bit
 * first; may be NULL only if D = 1.  Transcript: header "zkrelu_at" (log2 D, Q, R, has_GA,
 * 1), then "u" with the SHA-256 digest of the 4 log2 D x 32 point bytes; only u_bin is
 * drawn; from the claims on as zkrelu_prove.  Word 5 of the proof header is 1.  points_out
 * starts with the four given points.  ZKDL_EINVAL for a coordinate that is not below r. */
int zkrelu_prove_at(zkdl_ctx* ctx, const int64_t* Z, const int64_t* GA, uint64_t D, int Q, int R,
                    int src_on_device, const zkdl_fr* points, zkdl_transcript* tr, uint8_t* proof,
                    size_t* proof_len, zkdl_fr* claims, zkdl_fr* points_out, size_t* npoints);

/* One aggregation window of an L-layer width x width FCNN (Example FCNN,
 * Protocol zkdl): T' steps, stack slot n = t L + (l-1), N = T' L.  All five
 * stacks are device memory, row-major:
 *   A  int32 [N,B,width]      input of layer l
 *   W  int32 [N,width,width]  weights of layer l at step t
 *   GZ int32 [N,B,width]      gradient of Z^(l)
 *   Zr int64 [N,B,width]      Z^(l) where a ReLU follows, zero in last-layer slots
 *   GA int64 [N,B,width]      unscaled gradient of A^(l), zero in last-layer slots */
typedef struct {
    uint32_t L, B, width, T, Q, R;
    const int32_t* A;
    const int32_t* W;
    const int32_t* GZ;
    const int64_t* Zr;
    const int64_t* GA;
} zkdl_fcnn_witness;

/* What a window's proof leaves to be opened against commitments (Protocol zkdl, the proof-of-
 * evaluation line): claims "the multilinear extension of tensor T at point p is y".  A point is given
 * by reference into points_out: the concatenation of points_out[seg_off[s] .. seg_off[s] + seg_len[s])
 * for s < nseg, in the tensor's own axis order (stack index, rows, columns; for aux: slice k, row,
 * bit).  Stacks have N = T' L slots, slot n = t L + (l-1). */
typedef enum {
    ZKDL_T_A = 0,        /* A  [N,B,width]: input of layer l */
    ZKDL_T_W = 1,        /* W  [N,width,width] */
    ZKDL_T_GZ = 2,       /* GZ [N,B,width]: gradient of Z^(l) */
    ZKDL_T_Z = 3,        /* Z = A W of every layer [N,B,width] (the forward family's product) */
    ZKDL_T_ZR = 4,       /* Zr: Z where a ReLU follows, zero in last-layer slots (zkReLU's input) */
    ZKDL_T_GA = 5,       /* GA [N,B,width]: the gradA family's product = zkReLU's second input */
    ZKDL_T_GW = 6,       /* GW = A^T GZ [N,width,width] (the gradW family's product) */
    ZKDL_T_A_RELU = 7,   /* ReLU outputs (1 - sign) Z', slot (t,l) = input of layer l+1, zero in last-layer slots */
    ZKDL_T_GZ_RELU = 8,  /* (1 - sign) G_A': GZ with the last-layer slots zero */
    ZKDL_T_GZ_NEXT = 9,  /* GZ with slot (t,l) <- slot (t,l+1), zero in last-layer slots */
    ZKDL_T_W_NEXT = 10,  /* W with slot (t,l) <- slot (t,l+1), zero in last-layer slots; point in W's (in, out) order */
    ZKDL_T_AUX = 11,     /* aux [2, N B width, J]: the bit decompositions of Zr and GA */
    ZKDL_T_Z_LAST = 12,  /* Z of the last layer [T',B,width] */
    ZKDL_T_GZ_LAST = 13, /* GZ of the last layer [T',B,width] */
    ZKDL_T_U = 14        /* update_prove: U = G_W / 2^R rounded to nearest, W_next = W - U */
} zkdl_claim_tensor;
#define ZKDL_CLAIM_MAX_SEGS 4
typedef struct {
    uint32_t tensor; /* zkdl_claim_tensor */
    uint32_t nseg;
    uint32_t seg_off[ZKDL_CLAIM_MAX_SEGS];
    uint32_t seg_len[ZKDL_CLAIM_MAX_SEGS];
    zkdl_fr value;
} zkdl_claim;
#define ZKDL_AGGREGATE_NCLAIMS 14
#define ZKDL_AGGREGATE_LINKED_NCLAIMS 7

/* aggregate_prove: forward (Z = A W), gradA (G_A = G_Z^(l+1) W^(l+1)T, last
 * slot of each step zero), gradW (G_W = A^T G_Z) matmul sumchecks and zkReLU on
 * (Zr, GA), in that order on one transcript.
 * claims_out (host, may be NULL; *nclaims = capacity on entry, ZKDL_AGGREGATE_NCLAIMS needed, else
 * ZKDL_ESMALL before anything runs): the claims the four sumchecks leave side by side, in proof order -
 * forward: Z at (w,u0,u1), A at (v_n,u0,v_i), W at (v_n,v_i,u1); gradA: GA at (w,u0,u1), GZ_NEXT at
 * (v_n,u0,v_i), W_NEXT at (v_n,u1,v_i); gradW: GW at (w,u0,u1), A at (v_n,v_i,u0), GZ at (v_n,v_i,u1);
 * zkReLU: ZR at u_Z, A_RELU at u_A, GA at u_GA, GZ_RELU at u_GZ, AUX at (k*, v, w*).
 * The segments index points_out, which must then be given as well (ZKDL_EINVAL otherwise). */
int aggregate_prove(zkdl_ctx* ctx, const zkdl_fcnn_witness* w, zkdl_transcript* tr, uint8_t* proof,
                    size_t* proof_len, zkdl_fr* points_out, size_t* npoints, zkdl_claim* claims_out,
                    size_t* nclaims);

/* update_prove: the parameter update of a training step (Sec. 5, Example FCNN, the last item of its list:
 * "parameter updates, based on the selected optimizer", a family of its own in Protocol zkdl).  The paper fixes
 * no optimizer; this entry point proves plain SGD on fixed-point weights with a power-of-two learning rate,
 *   W_next = W - U,   U = G_W / 2^R rounded to the nearest integer, halves away from zero,
 * for the D = 2^k entries of a gradient stack G_W (int64, host or device; |G_W| < 2^(Q+R-1), Q + R <= 63, else
 * ZKDL_ERANGE / ZKDL_EINVAL).  U = ReLU(rescale(G_W)) - ReLU(rescale(-G_W)) with zkReLU's rescaling (Sec. 3.1),
 * so the rounding is proved by zkReLU's forward half (App. A) on the stack Zu = [G_W; -G_W]:
 *   1. p is drawn over the D entries; the prover claims a0 = Au~(0,p), a1 = Au~(1,p), Au = ReLU(rescale(Zu));
 *      U~(p) = a0 - a1 is the value the verifier compares with W~(p) - W_next~(p);
 *   2. a multilinear extension is linear in each coordinate, so the two claims lie on a line: rho is drawn after
 *      they are absorbed and Au~(rho, p) = (1 - rho) a0 + rho a1 is the one claim that stands for both;
 *   3. u_Z is drawn over the 1 + log2 D variables of Zu and zkReLU runs at the given points u_A = (rho, p),
 *      u_Z (as zkrelu_prove_at inside a larger proof: mode 2); its claim on Zu gives
 *      G_W~(u_Z[1:]) = Zu~(u_Z) / (1 - 2 u_Z[0]).
 * claims_out (ZKDL_UPDATE_NCLAIMS entries, may be NULL): U at p, GW at u_Z[1:], AUX (the bits of Zu) at zkReLU's
 * merged point; segments index points_out as in aggregate_prove.  points_out: every challenge in draw order,
 * with the three copied points of zkReLU (u_A, and u_Z twice for the unused backward side) after u_Z.
 * Transcript: header "update" (log2 D, Q, R); draw p; "c" a0, a1; one draw of rho and u_Z; zkReLU.
 * Proof: "ZKUP", log2 D, Q, R, 0, 0, 0, 0; a0, a1; a "ZKRL" block. */
#define ZKDL_UPDATE_NCLAIMS 3
int update_prove(zkdl_ctx* ctx, const int64_t* GW, uint64_t D, int Q, int R, int src_on_device, zkdl_transcript* tr,
                 uint8_t* proof, size_t* proof_len, zkdl_fr* points_out, size_t* npoints, zkdl_claim* claims_out,
                 size_t* nclaims);

/* aggregate_prove_ft: aggregate_prove with the three matrix-product families in the optimized aggregated
 * form of App. B (Protocol tensor-op-aggr-optimized), each as in sumcheck_matmul_ft: the log2 N stack
 * rounds send f_t(0), f_t(1), f_t(2) and fold two tables (no table for beta~(w, .)), then the single
 * product's sumcheck follows; zkReLU as in aggregate_prove.  Transcript header "aggregate_ft" (L, B, width,
 * T', Q, R).  Proof: "ZKAF", L, B, width, T', Q, R, 0, three "ZKSF" blocks (forward, gradA, gradW), the
 * zkReLU proof. */
int aggregate_prove_ft(zkdl_ctx* ctx, const zkdl_fcnn_witness* w, zkdl_transcript* tr, uint8_t* proof,
                       size_t* proof_len, zkdl_fr* points_out, size_t* npoints);

/* aggregate_prove_linked: the same four families with their claims chained (Sec. 3.2: the
 * claims zkReLU starts from are left by the other operations' sumchecks; Sec. 4, Eq.
 * sc-reindex: claims on stacks whose slots are shifted become claims on the stack itself;
 * Protocol zkdl, the sumcheck and re-indexing lines).  In order, on one transcript:
 *  1. forward, gradA, gradW as in aggregate_prove;
 *  2. zkReLU at u_Z = the point of forward's claim_0, u_A = the point of forward's final on
 *     A, u_GA = the point of gradA's claim_0, u_GZ = the point of gradW's final on G_Z
 *     (header "zkrelu_at" with mode 2: the points are not hashed again);
 *  3. re-indexing on A [N, B width] with two sub-stacks at forward's stack point v_n: A itself
 *     and the stack whose slot (t, l) is slot (t, l+1), zero for the last layer (the ReLU
 *     outputs), common point (u0, v_i);
 *  4. re-indexing on G_Z and on W with that shifted sub-stack alone, at gradA's stack point,
 *     common points (u0, v_i) and (u1, v_i);
 *  5. the two claims standing on A (from 3, and gradW's final on A^T) merged into one as in
 *     claims_merge_stack_prove, then the two on W (forward's final, and the one from 4).
 * One claim per stack is left.  The re-indexing and merge headers carry N, D, K only.  What the verifier checks between the parts
 * (c_GA = gradA's claim_0; forward's claim_0 - c_Z and gradW's final on G_Z - c_GZ are the
 * last layer's share; the sub-stack claims equal the finals and c_A) needs nothing from the
 * prover.  Proof: "ZKAL" header (L, B, width, T, Q, R, 0), three SC blocks, the zkReLU
 * proof, three "ZKRI" proofs, two "ZKMS" proofs.  points_out: every challenge in order; the 4 log2(N B width)
 * coordinates given to zkReLU are repeated in front of its own draws. */
/* claims_out (as for aggregate_prove; ZKDL_AGGREGATE_LINKED_NCLAIMS entries): the one claim per stack that is
 * left - A, W, GZ, Z_LAST, GZ_LAST, GW, AUX.  The values on Z_LAST and GZ_LAST are the last layer's share
 * divided by beta~ of the layer coordinates at L-1, as the verifier computes them (reported as zero in the
 * event, of probability about 2^-255 per coordinate, that this factor is zero). */
int aggregate_prove_linked(zkdl_ctx* ctx, const zkdl_fcnn_witness* w, zkdl_transcript* tr, uint8_t* proof,
                           size_t* proof_len, zkdl_fr* points_out, size_t* npoints, zkdl_claim* claims_out,
                           size_t* nclaims);

/* ---- verifier (Sec. 2.2: the round checks; App. A: the final claim of zkReLU; App. B: the verifier's side of
 * both aggregated protocols; Sec. 6: verification is sequential) ----
 * aggregate_verify replays, on the GPU (one block, the transcript steps shared out among its lanes), a proof of
 * aggregate_prove ("ZKAG"), aggregate_prove_ft ("ZKAF"), aggregate_prove_linked ("ZKAL"), update_prove ("ZKUP") or sumcheck_matmul_general ("ZKGA")
 * on the transcript `tr` as it stood before that call: it re-derives every challenge, checks every round
 * (g_t(0) + g_t(1) = claim, or (1 - w_t) f_t(0) + w_t f_t(1) = claim), every final claim (the recomputed
 * equality-polynomial values, the six zkReLU equations at the challenge point, the merge of the claims on aux,
 * the weights P~(v) of the re-indexings and of the merges), every link of a chained window (zkReLU's input claims
 * against the matrix products' claims, the sub-stack claims against the finals, each merge against the claims it
 * merges) and that every field element of the proof is canonical.
 * proof: host bytes.  *verdict = 0: accepted - the transcript is advanced to the state after the proof,
 * points_out / npoints receive the drawn challenges in draw order (without the repeats a prover's points_out
 * carries) and claims_out / nclaims the claims left to open (as aggregate_prove reports them; none for the other
 * forms, whose claims the caller reads from the prover's list).  *verdict != 0: rejected, 100 x stage + detail
 * (stage 1 header, 2 forward, 3 gradA, 4 gradW, 5 zkReLU, 6 its merge, 7 a link of a chained window, 8 - 10 the
 * re-indexings of A, G_Z, W, 11 - 12 the merges on A and W, 13 - 17 the parts of an update proof, 18 the general
 * aggregated form); the transcript
 * is untouched.  The return value is ZKDL_OK whenever the verification ran.  zkdl_host_aggregate_verify: the same
 * program compiled for the CPU. */
int aggregate_verify(zkdl_ctx* ctx, const uint8_t* proof, size_t proof_len, zkdl_transcript* tr, int* verdict,
                     zkdl_fr* points_out, size_t* npoints, zkdl_claim* claims_out, size_t* nclaims);
int zkdl_host_aggregate_verify(const uint8_t* proof, size_t proof_len, zkdl_transcript* tr, int* verdict,
                               zkdl_fr* points_out, size_t* npoints, zkdl_claim* claims_out, size_t* nclaims);

/* ---- commitments (Sec. 2.3; Sec. 1.1; Protocol zkdl, the commit and proof-of-evaluation lines) ----
 * Pedersen commitments in G1 of BLS12-381 (y^2 = x^3 + 4 over F_q, the subgroup of order r),
 *   Commit(S; rho) = rho H + sum_i S_i G_i,
 * and the row-wise commitment of a tensor: 2^m entries laid out as R = 2^ceil(m/2) rows of C = 2^floor(m/2)
 * columns (row index = the leading variables), row j committed with the generators G_0..G_{C-1} and its own
 * blinding rho_j, so that the commitment has O(sqrt(size)) group elements.
 * A group element crosses the boundary as 96 bytes: affine x then y, 48 bytes little-endian each, fully
 * reduced, not in Montgomery form; the identity as 96 zero bytes.
 *
 * zkdl_commit_key_create: the C = ncols generators and H of `label` (NUL-terminated, at most 16 bytes) and
 * their window tables, in device memory.  Generator i: for ctr = 0, 1, .. the candidate
 * x = int_be(SHA256(tag || u32be(i) || u32be(ctr) || 0x00) || SHA256(.. || 0x01)) mod q with
 * tag = "zkdl-mi355x/g1/" || label; the first x for which x^3 + 4 is a square gives (x, y) with the smaller
 * root y, multiplied by the cofactor (a candidate that becomes the identity is skipped); H is index
 * 0xFFFFFFFF.  ncols a power of two up to 2^15; max_bits 32 or 64: the widest tensor entry the key serves
 * (the tables hold the 2^w - 1 non-zero multiples per w-bit window and generator in affine form, 96 B each,
 * ceil(max_bits / w) windows: w = 12, 1.2 MB per generator at 32 bits, while that stays below 16 GiB for the
 * key, else w = 8, 98 KB per generator; zkdl_ctx_set_commit_window_bits).
 * zkdl_commit_key_generators: generators first .. first + count - 1 (index ncols = H) as bytes, for checks. */
typedef struct zkdl_commit_key zkdl_commit_key;
int zkdl_commit_key_create(zkdl_ctx* ctx, const char* label, uint64_t ncols, int max_bits, zkdl_commit_key** out);
int zkdl_commit_key_destroy(zkdl_ctx* ctx, zkdl_commit_key* key);
int zkdl_commit_key_generators(zkdl_ctx* ctx, const zkdl_commit_key* key, uint64_t first, uint64_t count,
                               uint8_t* host_out);
/* hyrax_commit: the R row commitments of X, an int32 or int64 tensor view (zkdl_tensor_wrap_int) of 2^m
 * entries with C <= the key's ncols (int64 needs a key made with max_bits = 64); a negative entry x is the
 * field element r - |x|, i.e. contributes -|x| G_i.  blind (host, R canonical elements, or NULL for zero
 * blinding).  commitments_out (host, R x 96 bytes); *ncommit = capacity in elements on entry, R on return
 * (ZKDL_ESMALL with *ncommit = R if too small). */
int hyrax_commit(zkdl_ctx* ctx, const zkdl_commit_key* key, const zkdl_tensor* X, const zkdl_fr* blind,
                 uint8_t* commitments_out, size_t* ncommit);
/* hyrax_open: the prover's message of the proof of evaluation of X~ at `point` (host, m canonical
 * elements, row coordinates first): T = sum_j beta~(v_row, j) X[j, :] (T_out, C elements),
 * rho* = sum_j beta~(v_row, j) rho_j (rho_out, may be NULL) and y = <T, beta~(v_col, .)> = X~(point).
 * The verifier combines the row commitments with the same weights (the homomorphism of Sec. 2.3) and
 * checks Commit(T; rho*) against the result and y against T.  X: any tensor of 2^m entries. */
int hyrax_open(zkdl_ctx* ctx, const zkdl_tensor* X, const zkdl_fr* blind, const zkdl_fr* point, size_t npoint,
               zkdl_fr* T_out, zkdl_fr* rho_out, zkdl_fr* y_out);

/* hyrax_verify: the verifier's side of that proof of evaluation (Sec. 2.3, the homomorphism; Protocol zkdl, the
 * proof-of-evaluation line): C* = sum_j beta~(v_row, j) C_j over the nrows row commitments (host, 96 bytes
 * each), Commit(T; rho*) on the key's generators, and <T, beta~(v_col, .)> against y.  point: npoint = log2 nrows
 * + log2 C canonical elements, row coordinates first; T: C elements; rho: rho* or NULL for zero blinding.
 * *verdict = 0 accepted, 1 malformed input (an element not below r, a commitment that is not an element of the
 * group of order r Sec. 2.3 works in: off the curve, or on it but outside the subgroup), 2 the opened row does not
 * match the combined commitment, 3 wrong evaluation.  combined_out (may be NULL): C* as 96 bytes; without it the
 * two sums are compared as projective points and no inversion is taken.
 * Both sums run on the GPU, eight lanes per term (every point operation shared by the eight; a scalar split in
 * two halves of 128 bits by the curve's endomorphism, 4-bit windows), next to the membership test of the
 * commitments; the weights, the split and the inner product on the host. */
int hyrax_verify(zkdl_ctx* ctx, const zkdl_commit_key* key, const uint8_t* commitments, size_t nrows,
                 const zkdl_fr* point, size_t npoint, const zkdl_fr* T, const zkdl_fr* rho, const zkdl_fr* y,
                 int* verdict, uint8_t* combined_out);

/* Re-derives the constants of the base-field arithmetic on the host and checks the unreduced point additions, the
 * endomorphism's constant and the split of a scalar against plain computations; ZKDL_OK if they match. */
int zkdl_commit_selfcheck(void);

/* ---- per-kernel timing (for callers that measure; paper-independent) -------
 * While enabled, the launches of the kernel classes below are bracketed by HIP
 * events on the context's stream; zkdl_ctx_profile_read returns, per class and
 * since the last reset, the number of launches, the summed event time in ms and
 * the summed algorithmic bytes (bytes the operation must read and write, not
 * what the memory system moved). */
#define ZKDL_PROF_SC_ROUND_FUSED 0 /* fused fold-and-evaluate sumcheck round */
#define ZKDL_PROF_SC_ROUND_FIRST 1 /* first sumcheck round (evaluate only) */
#define ZKDL_PROF_PARTIAL_EVAL 2   /* beta-weighted axis contraction */
#define ZKDL_PROF_ZK_BIN 3         /* zkReLU binarity rounds on the D x (Q+R) tables */
#define ZKDL_PROF_ZK_LIN 4         /* zkReLU linear rounds on the D-sized tables */
#define ZKDL_PROF_FINALISE 5       /* per-round transcript step */
#define ZKDL_PROF_CLASSES 6
int zkdl_ctx_profile_enable(zkdl_ctx* ctx, int on);
int zkdl_ctx_profile_reset(zkdl_ctx* ctx);
int zkdl_ctx_profile_read(zkdl_ctx* ctx, int cls, uint64_t* launches, double* total_ms,
                          double* total_bytes);

/* ---- machine probes (for callers that report roofline fractions; paper-independent) ----
 * Runs one probe kernel on the context's stream (after an untimed warm-up launch) and returns the
 * work it did and the time HIP events measured around it:
 *   ZKDL_SB_COPY    a device-to-device copy of `work` bytes (multiple of 16, at most 2^34);
 *                   *units = bytes read + bytes written = 2 work
 *   ZKDL_SB_MAD     2048 blocks x 256 threads, each running `work` x 64 multiply-adds of 32 x 32 + 64
 *                   bits in 16 independent register chains; *units = multiply-adds
 *   ZKDL_SB_MODMUL  the same grid, each thread `work` x 2 Montgomery products of the field
 *                   multiplier in registers; *units = products
 * work <= 2^24 for the last two.  The copy takes its two buffers from the context's allocator. */
#define ZKDL_SB_COPY 0
#define ZKDL_SB_MAD 1
#define ZKDL_SB_MODMUL 2
int zkdl_selfbench(zkdl_ctx* ctx, int what, uint64_t work, double* units, double* seconds);

/* ---- host-side self checks (no GPU needed) -------------------------------- */
/* out = a * b mod r computed by the library's Montgomery code on the host. */
int zkdl_host_fr_mul(const zkdl_fr* a, const zkdl_fr* b, zkdl_fr* out);
/* Re-derives the Montgomery constants by modular doubling; ZKDL_OK if they match. */
int zkdl_selfcheck_constants(void);
/* The split of a scalar that hyrax_verify hands to its kernels: k (32 bytes little-endian, any value) =
 * a + b z^2 with z^2 = 0xd201000000010000^2 and a < z^2; out = a (16 bytes little-endian) then b (16 bytes).
 * ZKDL_EINVAL if b does not fit 128 bits (k >= 2^128 z^2; never for k below r). */
int zkdl_host_scalar_split(const zkdl_fr* k, uint8_t out[32]);

#ifdef __cplusplus
}
#endif
#endif /* ZKDL_H */
