// aggregate_verify: the verifier of an aggregated window on the GPU (Sec. 6 names verification time as the
// open problem: it is sequential).  The program of verify.cuh runs in one block; the host only moves the
// proof in and the verdict, the challenges and the transcript state out.  zkdl_host_aggregate_verify runs the
// same program on the CPU (used by the library's tests without a GPU).
#include <string.h>
#include <new>

#include "zkdl_internal.h"
#include "verify.cuh"

namespace {

constexpr int VERIFY_STAGE_BYTES = 32768;

struct VerifyOut {
    int verdict;
    int n_chal;
    ts::State s;
};

// One block: every thread runs the same sequential program (same branches: the proof decides them); the
// transcript steps are shared out among the lanes as in the prover's kernels.  The challenges go to st->chal
// and, canonical, to st->chal_le as they are drawn.
__global__ __launch_bounds__(ZK_BLOCK) void k_verify_aggregate(const uint8_t* proof, uint64_t len, ts::State s0, DevState* st,
                                                               VerifyOut* out) {
    __shared__ TsShared S;
    __shared__ vf::DevShared D;
    __shared__ uint32_t staged[VERIFY_STAGE_BYTES / 4];   // the proof, when it fits: every later read is an LDS read
    const int tid = threadIdx.x;
    if (len <= (uint64_t)VERIFY_STAGE_BYTES) {
        const uint32_t nw = (uint32_t)((len + 3) / 4);   // the buffer is padded to a multiple of 256 bytes
        for (uint32_t i = tid; i < nw; i += blockDim.x) staged[i] = ((const uint32_t*)proof)[i];
        proof = (const uint8_t*)staged;
    }
    if (tid < 8) S.state[tid] = s0.h[tid];
    if (tid >= 16 && tid < 32) {
        uint32_t w = 0;
        for (int b = 0; b < 4; ++b) {
            const uint32_t at = 4u * (uint32_t)(tid - 16) + (uint32_t)b;
            w = (w << 8) | (at < s0.fill ? (uint32_t)s0.buf[at] : 0u);
        }
        S.buf[0][tid - 16] = w;
    }
    if (tid == 8) {
        S.nblk = s0.nblk;
        S.fill = s0.fill;
        S.bufsel = 0;
    }
    __syncthreads();
    vf::DevCtx c;
    c.chal = st->chal;
    c.n_chal = 0;
    c.inv2 = st->inv2;
    c.inv6 = st->inv6;
    c.overflow = false;
    c.S = &S;
    c.D = &D;
    c.st = st;
    const int verdict = vf::aggregate(c, proof, (size_t)len);
    __syncthreads();
    if (tid == 0) {
        out->verdict = verdict;
        out->n_chal = c.n_chal;
        for (int i = 0; i < 8; ++i) out->s.h[i] = S.state[i];
        out->s.nblk = S.nblk;
        out->s.fill = S.fill;
        for (uint32_t i = 0; i < 64; ++i)
            out->s.buf[i] = i < S.fill ? (uint8_t)(S.buf[S.bufsel][i >> 2] >> (24 - 8 * (i & 3))) : (uint8_t)0;
    }
}

// offsets of the four parts of a "ZKAG" proof and their first challenge indices, from the header
bool unlinked_layout(const uint8_t* proof, size_t len, uint32_t hdr[8], int c[4], size_t p[5]) {
    if (len < 32) return false;
    for (int i = 0; i < 8; ++i)
        hdr[i] = (uint32_t)proof[4 * i] | ((uint32_t)proof[4 * i + 1] << 8) | ((uint32_t)proof[4 * i + 2] << 16) |
                 ((uint32_t)proof[4 * i + 3] << 24);
    if (hdr[0] != vf::ZKAG_MAGIC) return false;
    const int ln = vf::ilog2((uint64_t)hdr[1] * hdr[4]), lb = vf::ilog2(hdr[2]), lw = vf::ilog2(hdr[3]);
    if (ln < 0 || lb < 0 || lw < 0) return false;
    auto sc = [](int rounds) { return (size_t)16 + 32 + (size_t)rounds * 128 + 96; };
    p[0] = 32;
    p[1] = p[0] + sc(ln + lw);
    p[2] = p[1] + sc(ln + lw);
    p[3] = p[2] + sc(ln + lb);
    p[4] = len;
    c[0] = 0;
    c[1] = c[0] + (ln + lb + lw) + (ln + lw);
    c[2] = c[1] + (ln + lb + lw) + (ln + lw);
    c[3] = c[2] + (ln + lw + lw) + (ln + lb);
    return p[3] < len;
}

int finish_verify(zkdl_transcript* tr, int verdict_in, const ts::State& s_after, int n_chal, const uint8_t* chal_le,
                  const uint8_t* proof, size_t proof_len, int* verdict, zkdl_fr* points_out, size_t* npoints,
                  zkdl_claim* claims_out, size_t* nclaims) {
    *verdict = verdict_in;
    if (npoints) {
        const size_t cap = *npoints;
        *npoints = (size_t)n_chal;
        if (points_out && cap < (size_t)n_chal) return ZKDL_ESMALL;
    }
    if (verdict_in != 0) {   // rejected: nothing of the caller's changes
        if (nclaims) *nclaims = 0;
        return ZKDL_OK;
    }
    if (points_out && npoints) memcpy(points_out, chal_le, 32 * (size_t)n_chal);
    if (claims_out && nclaims) {
        uint32_t hdr[8];
        int c[4];
        size_t p[5];
        if (unlinked_layout(proof, proof_len, hdr, c, p)) {
            if (*nclaims < ZKDL_AGGREGATE_NCLAIMS) {
                *nclaims = ZKDL_AGGREGATE_NCLAIMS;
                return ZKDL_ESMALL;
            }
            *nclaims = zk_claims_unlinked(claims_out, proof, hdr[1], hdr[2], hdr[3], hdr[4], hdr[5], hdr[6], c[0], p[0], c[1],
                                          p[1], c[2], p[2], c[3], p[3], p[4]);
        } else {
            *nclaims = 0;   // the f_t form: its claims are read from the proof by the caller
        }
    }
    tr->s = s_after;
    return ZKDL_OK;
}

}  // namespace

extern "C" int zkdl_host_aggregate_verify(const uint8_t* proof, size_t proof_len, zkdl_transcript* tr, int* verdict,
                                          zkdl_fr* points_out, size_t* npoints, zkdl_claim* claims_out, size_t* nclaims) {
    if (!proof || !tr || !verdict) return ZKDL_EINVAL;
    Fr* chal = new (std::nothrow) Fr[vf::MAX_CHAL];
    uint8_t* le = new (std::nothrow) uint8_t[32 * vf::MAX_CHAL];
    if (!chal || !le) {
        delete[] chal;
        delete[] le;
        return ZKDL_ENOMEM;
    }
    ts::State live = tr->s;
    vf::HostCtx c;
    c.chal = chal;
    c.n_chal = 0;
    c.overflow = false;
    c.s = &live;
    vf::host_inverses(c.inv2, c.inv6);
    const int v = vf::aggregate(c, proof, proof_len);
    for (int i = 0; i < c.n_chal; ++i) ts::fr_to_le(chal[i], le + 32 * (size_t)i);
    const int rc = finish_verify(tr, v, live, c.n_chal, le, proof, proof_len, verdict, points_out, npoints, claims_out, nclaims);
    delete[] chal;
    delete[] le;
    return rc;
}

extern "C" int aggregate_verify(zkdl_ctx* ctx, const uint8_t* proof, size_t proof_len, zkdl_transcript* tr, int* verdict,
                                zkdl_fr* points_out, size_t* npoints, zkdl_claim* claims_out, size_t* nclaims) {
    if (!ctx || !proof || !tr || !verdict || proof_len == 0 || proof_len > (size_t)ZK_PROOF_CAP) return ZKDL_EINVAL;
    ZK_HIP(ctx, hipSetDevice(ctx->device));
    uint8_t* d_proof = (uint8_t*)zk_alloc(ctx, proof_len);   // 256-byte aligned: the kernel reads whole words
    VerifyOut* d_out = (VerifyOut*)zk_alloc(ctx, sizeof(VerifyOut));
    int rc = (d_proof && d_out) ? ZKDL_OK : ZKDL_ENOMEM;
    VerifyOut h_out;
    memset(&h_out, 0, sizeof h_out);
    uint8_t* h_le = ctx->host_stage;   // pinned; 32 KiB of it
    static_assert(sizeof(DevState) >= 32 * vf::MAX_CHAL, "staging buffer holds the challenges");
    static_assert(vf::MAX_CHAL <= ZK_MAX_CHAL, "the state block holds the verifier's challenges");
    hipError_t e = hipSuccess;
    if (rc == ZKDL_OK) {
        e = hipMemcpyAsync(d_proof, proof, proof_len, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) {
            hipLaunchKernelGGL(k_verify_aggregate, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, d_proof, (uint64_t)proof_len, tr->s,
                               ctx->dev, d_out);
            e = hipMemcpyAsync(&h_out, d_out, sizeof h_out, hipMemcpyDeviceToHost, ctx->stream);
        }
        if (e == hipSuccess)
            e = hipMemcpyAsync(h_le, ctx->dev->chal_le, 32 * vf::MAX_CHAL, hipMemcpyDeviceToHost, ctx->stream);
    }
    hipError_t e2 = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess) e = e2;
    if (e == hipSuccess) e = hipGetLastError();
    zk_free(ctx, d_proof);
    zk_free(ctx, d_out);
    if (rc != ZKDL_OK) return rc;
    ZK_HIP(ctx, e);
    return finish_verify(tr, h_out.verdict, h_out.s, h_out.n_chal, h_le, proof, proof_len, verdict, points_out, npoints, claims_out,
                         nclaims);
}
