// Machine probes behind the C ABI (zkdl_selfbench): the rates that a kernel's roofline fractions
// are quoted against, measured on the GPU the context runs on instead of taken from a datasheet.
//  - a plain device-to-device copy (what the memory system sustains for a streaming kernel);
//  - a register-only loop of independent v_mad_u64_u32 chains (the 32 x 32 + 64-bit multiply-add
//    that the field multiplier is made of);
//  - a register-only loop of the library's own Montgomery product on 29-bit limbs (f9_mul).
// None of them is part of a proof.
#include "zkdl_internal.h"

// ---- copy: 16 bytes per thread and step, grid-stride ----
__global__ __launch_bounds__(ZK_BLOCK) void k_sb_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, uint64_t n16) {
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n16; i += (uint64_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

// ---- multiply-add: SB_CHAINS independent chains per thread, each acc <- lo32(acc) * m + acc ----
constexpr int SB_CHAINS = 16;
constexpr int SB_UNROLL = 4;

__global__ __launch_bounds__(ZK_BLOCK) void k_sb_mad(uint32_t iters, uint32_t seed, uint64_t* out) {
    uint64_t acc[SB_CHAINS];
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t m = (seed ^ gid) | 1u;
#pragma unroll
    for (int j = 0; j < SB_CHAINS; ++j) acc[j] = ((uint64_t)gid << 20) + (uint64_t)(j + 1) * seed;
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < SB_UNROLL; ++u) {
#pragma unroll
            for (int j = 0; j < SB_CHAINS; ++j) acc[j] = (uint64_t)(uint32_t)acc[j] * m + acc[j];
        }
    }
    uint64_t s = 0;
#pragma unroll
    for (int j = 0; j < SB_CHAINS; ++j) s ^= acc[j];
    out[gid] = s;   // one store per thread keeps the chains alive
}

// ---- Montgomery product in registers: two independent chains x <- x * y per thread ----
__global__ __launch_bounds__(ZK_BLOCK) void k_sb_modmul(uint32_t iters, uint32_t seed, uint32_t* out) {
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    F9 x0, x1, y;
#pragma unroll
    for (int l = 0; l < 9; ++l) {
        x0.v[l] = (seed * (uint32_t)(l + 3) + gid) & frc::M29;
        x1.v[l] = (seed * (uint32_t)(l + 7) ^ gid) & frc::M29;
        y.v[l] = (seed + 977u * (uint32_t)l + gid * 31u) & frc::M29;
    }
    // values below 2^256 keep every product normal and below 2^256 (f9_mul: a b / 2^261 + r)
    x0.v[8] &= 0xffffffu;
    x1.v[8] &= 0xffffffu;
    y.v[8] &= 0xffffffu;
    for (uint32_t it = 0; it < iters; ++it) {
        x0 = f9_mul(x0, y);
        x1 = f9_mul(x1, y);
    }
    uint32_t s = 0;
#pragma unroll
    for (int l = 0; l < 9; ++l) s ^= x0.v[l] ^ x1.v[l];
    out[gid] = s;
}

extern "C" int zkdl_selfbench(zkdl_ctx* ctx, int what, uint64_t work, double* units, double* seconds) {
    if (!ctx || !units || !seconds || work == 0) return ZKDL_EINVAL;
    ZK_HIP(ctx, hipSetDevice(ctx->device));
    hipEvent_t e0, e1;
    ZK_HIP(ctx, hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return ZKDL_EHIP;
    }
    int rc = ZKDL_OK;
    void *a = nullptr, *b = nullptr;
    const unsigned grid = 256 * 8;   // eight blocks of four waves on each of the 256 compute units
    double done = 0.0;
    if (what == ZKDL_SB_COPY) {
        if (work % 16 != 0 || work > ((uint64_t)1 << 34)) {
            rc = ZKDL_EINVAL;
        } else {
            a = zk_alloc(ctx, work);
            b = zk_alloc(ctx, work);
            if (!a || !b) rc = ZKDL_ENOMEM;
        }
        if (rc == ZKDL_OK) {
            (void)hipMemsetAsync(a, 1, work, ctx->stream);
            const uint64_t n16 = work / 16;
            uint64_t want = (n16 + ZK_BLOCK - 1) / ZK_BLOCK;
            const unsigned g = (unsigned)(want < 256 * 32 ? (want ? want : 1) : 256 * 32);
            hipLaunchKernelGGL(k_sb_copy, dim3(g), dim3(ZK_BLOCK), 0, ctx->stream, (const uint4*)a, (uint4*)b, n16);
            (void)hipEventRecord(e0, ctx->stream);
            hipLaunchKernelGGL(k_sb_copy, dim3(g), dim3(ZK_BLOCK), 0, ctx->stream, (const uint4*)a, (uint4*)b, n16);
            (void)hipEventRecord(e1, ctx->stream);
            done = 2.0 * (double)work;   // bytes read + bytes written
        }
    } else if (what == ZKDL_SB_MAD || what == ZKDL_SB_MODMUL) {
        if (work > ((uint64_t)1 << 24)) rc = ZKDL_EINVAL;
        a = rc == ZKDL_OK ? zk_alloc(ctx, (size_t)grid * ZK_BLOCK * 8) : nullptr;   // one result word per thread
        if (rc == ZKDL_OK && !a) rc = ZKDL_ENOMEM;
        if (rc == ZKDL_OK) {
            const uint32_t iters = (uint32_t)work;
            for (int pass = 0; pass < 2; ++pass) {   // the first launch warms up, the second is timed
                if (pass == 1) (void)hipEventRecord(e0, ctx->stream);
                if (what == ZKDL_SB_MAD)
                    hipLaunchKernelGGL(k_sb_mad, dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, iters, 0x9e3779b9u, (uint64_t*)a);
                else
                    hipLaunchKernelGGL(k_sb_modmul, dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, iters, 0x9e3779b9u, (uint32_t*)a);
            }
            (void)hipEventRecord(e1, ctx->stream);
            const double threads = (double)grid * ZK_BLOCK;
            done = what == ZKDL_SB_MAD ? threads * iters * SB_UNROLL * SB_CHAINS : threads * iters * 2.0;
        }
    } else {
        rc = ZKDL_EINVAL;
    }
    hipError_t e = hipStreamSynchronize(ctx->stream);
    float ms = 0.f;
    if (rc == ZKDL_OK && e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (rc == ZKDL_OK && e == hipSuccess) e = hipGetLastError();
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    zk_free(ctx, a);
    zk_free(ctx, b);
    if (rc != ZKDL_OK) return rc;
    ZK_HIP(ctx, e);
    *units = done;
    *seconds = (double)ms * 1e-3;
    return ZKDL_OK;
}
