// Base-threshold calibration: exact nearest-rank quantile of the pooled prefix
// magnitudes (the percentile stand-in for the error-bounded search of section
// 3.2.2) by radix select on the fp32 bit patterns.  Non-negative floats order
// like their unsigned bit patterns, so three histogram passes over bits
// [30:20], [19:9], [8:0] pin down the k-th smallest value exactly.  All integer
// work; integer atomics commute, so the result does not depend on scheduling.
#include <math.h>

#include "clada_internal.h"

namespace {

constexpr int NBINS = 2048;
constexpr int NPASS = 3;
__constant__ const int c_shift[NPASS] = {20, 9, 0};
__constant__ const int c_bits[NPASS] = {11, 11, 9};

struct CalibState {
    unsigned long long hist[NPASS][NBINS];
    unsigned long long k;        // remaining 1-based rank inside the current prefix
    unsigned int prefix;         // bits fixed so far
    unsigned int prefix_mask;
};

__global__ void __launch_bounds__(256) k_calib_init(CalibState *st, unsigned long long k)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < NPASS * NBINS) (&st->hist[0][0])[i] = 0ull;
    if (i == 0) {
        st->k = k;
        st->prefix = 0u;
        st->prefix_mask = 0u;
    }
}

// The magnitudes crowd into a few dozen bins (pass 0 sees mostly exponent bits), and LDS atomics
// of a wave to one address are served one lane at a time.  The workgroup therefore keeps 16
// histogram copies, chosen by lane % 16 (at most four lanes of a wave share an address), each
// shifted by one bank so that the copies of one bin do not collide either; 128 KiB of LDS, one
// workgroup of 1024 threads per compute unit, four 16-byte loads in flight per thread.
constexpr int HIST_COPIES = 16;
constexpr int HIST_PITCH = NBINS + 1;
constexpr int CALIB_THREADS = 1024;
__global__ void __launch_bounds__(CALIB_THREADS)
k_calib_hist(const float *__restrict__ pool, long long n, CalibState *st, int pass)
{
    __shared__ unsigned int s_hist[HIST_COPIES * HIST_PITCH];
    for (int i = threadIdx.x; i < HIST_COPIES * HIST_PITCH; i += CALIB_THREADS) s_hist[i] = 0u;
    __syncthreads();
    unsigned int *mine = s_hist + (threadIdx.x & (HIST_COPIES - 1)) * HIST_PITCH;
    const unsigned int prefix = st->prefix, pmask = st->prefix_mask;
    const int shift = c_shift[pass];
    const unsigned int dmask = (1u << c_bits[pass]) - 1u;
    const long long n4 = n >> 2;
    const u32x4 *p4 = reinterpret_cast<const u32x4 *>(pool);
    const long long stride = (long long)gridDim.x * CALIB_THREADS;
    auto count = [&](const u32x4 v) {
        const unsigned int u[4] = {v.x & 0x7fffffffu, v.y & 0x7fffffffu, v.z & 0x7fffffffu, v.w & 0x7fffffffu};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if ((u[e] & pmask) == prefix) atomicAdd(&mine[(u[e] >> shift) & dmask], 1u);
    };
    long long i = (long long)blockIdx.x * CALIB_THREADS + threadIdx.x;
    for (; i + 3 * stride < n4; i += 4 * stride) {
        u32x4 v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = __builtin_nontemporal_load(p4 + i + r * stride);
#pragma unroll
        for (int r = 0; r < 4; ++r) count(v[r]);
    }
    for (; i < n4; i += stride) count(__builtin_nontemporal_load(p4 + i));
    if (blockIdx.x == 0) {
        const unsigned int *p1 = reinterpret_cast<const unsigned int *>(pool);
        for (long long t = (n4 << 2) + threadIdx.x; t < n; t += CALIB_THREADS) {
            const unsigned int u = p1[t] & 0x7fffffffu;
            if ((u & pmask) == prefix) atomicAdd(&mine[(u >> shift) & dmask], 1u);
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < NBINS; b += CALIB_THREADS) {
        unsigned int c = 0u;
#pragma unroll
        for (int h = 0; h < HIST_COPIES; ++h) c += s_hist[h * HIST_PITCH + b];
        if (c) atomicAdd(&st->hist[pass][b], (unsigned long long)c);
    }
}

// Pick the bin that holds rank k, descend into it.
__global__ void __launch_bounds__(256) k_calib_select(CalibState *st, int pass, float *tau_out)
{
    __shared__ unsigned long long s_seg[256];
    const int tid = threadIdx.x;
    constexpr int PER = NBINS / 256;
    unsigned long long loc[PER], sum = 0ull;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        loc[e] = st->hist[pass][tid * PER + e];
        sum += loc[e];
    }
    s_seg[tid] = sum;
    __syncthreads();
    if (tid == 0) {
        unsigned long long k = st->k, run = 0ull;
        int seg = 255;
        for (int t = 0; t < 256; ++t) {
            if (run + s_seg[t] >= k) { seg = t; break; }
            run += s_seg[t];
        }
        int bin = seg * PER + PER - 1;
        for (int e = 0; e < PER; ++e) {
            const unsigned long long c = st->hist[pass][seg * PER + e];
            if (run + c >= k) { bin = seg * PER + e; break; }
            run += c;
        }
        const unsigned int dmask = (1u << c_bits[pass]) - 1u;
        st->k = k - run;
        st->prefix |= (unsigned int)bin << c_shift[pass];
        st->prefix_mask |= dmask << c_shift[pass];
        if (pass == NPASS - 1) *tau_out = __uint_as_float(st->prefix);
    }
}

}  // namespace

size_t clada_ws_calibrate(void) { return align_up(sizeof(CalibState), 256); }

extern "C" clada_status clada_threshold_calibrate(clada_ctx *ctx, const float *abs_act_pool, int64_t n,
                                                  float target_sparsity, float *tau_base_out,
                                                  void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    if (!abs_act_pool || !tau_base_out) return clada_fail(ctx, CLADA_ERR_NULL, "pool or output is NULL");
    if (n < 1) return clada_fail(ctx, CLADA_ERR_SHAPE, "n=%lld must be >= 1", (long long)n);
    if (!(target_sparsity >= 0.0f) || !(target_sparsity < 1.0f))
        return clada_fail(ctx, CLADA_ERR_VALUE, "target_sparsity=%g outside [0,1)", (double)target_sparsity);
    if (!aligned16(abs_act_pool)) return clada_fail(ctx, CLADA_ERR_ALIGN, "pool must be 16-byte aligned");
    const size_t need = CLADA_WS_HEADER + clada_ws_calibrate();
    if (ctx->ws_bytes < need)
        return clada_fail(ctx, CLADA_ERR_WORKSPACE, "workspace %zu < %zu bytes needed", ctx->ws_bytes, need);
    // nearest rank, taken in fp64 on the fp32 value of q
    long long k = (long long)ceil((double)target_sparsity * (double)n);
    if (k < 1) k = 1;
    if (k > n) k = n;
    CalibState *st = reinterpret_cast<CalibState *>(ctx->ws + CLADA_WS_HEADER);
    hipStream_t stream = (hipStream_t)hip_stream;
    hipLaunchKernelGGL(k_calib_init, dim3((NPASS * NBINS + 255) / 256), dim3(256), 0, stream, st,
                       (unsigned long long)k);
    long long want = ((n >> 2) + 4 * CALIB_THREADS - 1) / (4 * CALIB_THREADS);
    const int cap = ctx->num_cu;
    const int blocks = (int)(want < 1 ? 1 : (want > cap ? cap : want));
    for (int pass = 0; pass < NPASS; ++pass) {
        hipLaunchKernelGGL(k_calib_hist, dim3(blocks), dim3(CALIB_THREADS), 0, stream, abs_act_pool, (long long)n, st, pass);
        hipLaunchKernelGGL(k_calib_select, dim3(1), dim3(256), 0, stream, st, pass, tau_base_out);
    }
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    return CLADA_OK;
}
