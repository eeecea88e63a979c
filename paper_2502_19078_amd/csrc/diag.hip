// Measurement helpers: a plain streaming-read kernel (the practical HBM ceiling the
// decode kernels are compared with) and a plain copy kernel (the known-size traffic
// against which the profiler's FETCH_SIZE / WRITE_SIZE counters are scaled).
#include "clada_internal.h"

namespace {

template <int UNROLL>
__global__ void __launch_bounds__(256)
k_stream_read(const u32x4 *__restrict__ src, size_t n16, unsigned int *__restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + (UNROLL - 1) * stride < n16; i += UNROLL * stride) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc ^= v[u];
    }
    for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    const unsigned int r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (r == 0x9e3779b9u) sink[blockIdx.x & 63] = r;   // practically never taken; keeps the loads alive
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
    if (!aligned16(src) || bytes % 16 != 0) return clada_fail(ctx, CLADA_ERR_ALIGN, "src/bytes must be multiples of 16");
    if (blocks_per_cu < 1 || blocks_per_cu > 32) return clada_fail(ctx, CLADA_ERR_VALUE, "blocks_per_cu outside [1,32]");
    if (ctx->ws_bytes == 0) return clada_fail(ctx, CLADA_ERR_WORKSPACE, "context has no device");
    hipLaunchKernelGGL(k_stream_read<8>, dim3(ctx->num_cu * blocks_per_cu), dim3(256), 0, (hipStream_t)hip_stream,
                       (const u32x4 *)src, bytes / 16, reinterpret_cast<unsigned int *>(ctx->ws + 2048));
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
