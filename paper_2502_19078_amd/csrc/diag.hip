// Measurement helpers: a plain streaming-read kernel (the practical HBM ceiling the
// decode kernels are compared with) and a plain copy kernel (the known-size traffic
// against which the profiler's FETCH_SIZE / WRITE_SIZE counters are scaled).
#include "clada_internal.h"

namespace {

// Whole-row streaming, the access pattern of the decode kernels: every wave reads 8 KiB rows
// (one 16-byte non-temporal load per lane per KiB), rows dealt round-robin over all waves.
__global__ void __launch_bounds__(512)
k_stream_read(const char *__restrict__ src, size_t nrows, unsigned int *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    const size_t gw = (size_t)blockIdx.x * 8 + (threadIdx.x >> 6), nw = (size_t)gridDim.x * 8;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t r = gw; r < nrows; r += nw) {
        const char *row = src + r * 8192 + lane * 16;
        u32x4 v[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row + c * 1024));
#pragma unroll
        for (int c = 0; c < 8; ++c) acc ^= v[c];
    }
    const unsigned int x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9e3779b9u) sink[blockIdx.x & 63] = x;   // practically never taken; keeps the loads alive
}

__global__ void __launch_bounds__(256)
k_copy(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace

extern "C" clada_status clada_diag_stream_read(clada_ctx *ctx, const void *src, size_t bytes,
                                               int32_t blocks_per_cu, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    if (!src) return clada_fail(ctx, CLADA_ERR_NULL, "src is NULL");
    if (!aligned16(src) || bytes % 8192 != 0) return clada_fail(ctx, CLADA_ERR_ALIGN, "src must be 16-byte aligned, bytes a multiple of 8192");
    if (blocks_per_cu < 1 || blocks_per_cu > 4) return clada_fail(ctx, CLADA_ERR_VALUE, "blocks_per_cu outside [1,4]");
    if (ctx->ws_bytes == 0) return clada_fail(ctx, CLADA_ERR_WORKSPACE, "context has no device");
    hipLaunchKernelGGL(k_stream_read, dim3(ctx->num_cu * blocks_per_cu), dim3(512), 0, (hipStream_t)hip_stream,
                       (const char *)src, bytes / 8192, reinterpret_cast<unsigned int *>(ctx->ws + 2048));
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    return CLADA_OK;
}

extern "C" clada_status clada_diag_copy(clada_ctx *ctx, const void *src, void *dst, size_t bytes, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    if (!src || !dst) return clada_fail(ctx, CLADA_ERR_NULL, "src or dst is NULL");
    if (!aligned16(src) || !aligned16(dst) || bytes % 16 != 0)
        return clada_fail(ctx, CLADA_ERR_ALIGN, "src/dst/bytes must be multiples of 16");
    if (ctx->ws_bytes == 0) return clada_fail(ctx, CLADA_ERR_WORKSPACE, "context has no device");
    hipLaunchKernelGGL(k_copy, dim3(ctx->num_cu * 8), dim3(256), 0, (hipStream_t)hip_stream,
                       (const u32x4 *)src, (u32x4 *)dst, bytes / 16);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    return CLADA_OK;
}
