// Cognitive-load signals (surprisal and entropy equations of section 2.3.1) and
// the token-aware threshold (final-threshold equation of section 3.2.3).
//
// Signals: one pass over the logits.  Every thread keeps an online triple
//   m = running max,  Z = sum e^{z-m},  T = sum e^{z-m} (z-m)
// so that  lse = m + log Z,  entropy = log Z - T/Z,  surprisal = lse - z_tok.
// Triples merge associatively (rescale by e^{m_i - m}); lanes merge by a fixed
// butterfly, waves through LDS, blocks through the workspace with the last
// arriving block of each row folding the block partials in a fixed order, so
// the result is bit-reproducible.
#include <math.h>

#include <mutex>

#include "clada_internal.h"

namespace {

struct Lse {
    float m, Z, T;
    int bad;   // saw NaN or +inf
};

__device__ __forceinline__ Lse lse_empty() { return Lse{-INFINITY, 0.0f, 0.0f, 0}; }

__device__ __forceinline__ Lse lse_merge(const Lse a, const Lse b)
{
    Lse r;
    r.bad = a.bad | b.bad;
    r.m = fmaxf(a.m, b.m);
    r.Z = 0.0f;
    r.T = 0.0f;
    if (a.Z > 0.0f) {
        const float dm = a.m - r.m, c = expf(dm);
        r.Z += c * a.Z;
        r.T += c * (a.T + dm * a.Z);
    }
    if (b.Z > 0.0f) {
        const float dm = b.m - r.m, c = expf(dm);
        r.Z += c * b.Z;
        r.T += c * (b.T + dm * b.Z);
    }
    return r;
}

template <int ES>
__device__ __forceinline__ float load_logit(const char *row, int v)
{
    if (ES == 4) return reinterpret_cast<const float *>(row)[v];
    return __uint_as_float((unsigned int)reinterpret_cast<const unsigned short *>(row)[v] << 16);
}

constexpr int SIG_THREADS = 256;
constexpr int SIG_GROUP = 8;                       // logits folded per online update
constexpr int SIG_CHUNK = SIG_THREADS * SIG_GROUP * 2;   // logits per block

// Optional tail of the signals kernel: the token-aware thresholds of all layers for the row just finished
// (final-threshold equation of section 3.2.3); L = 0 switches it off.
struct ThresholdTail {
    const float *tau_base, *lambda, *gamma;   // [L]
    float *tau_final;                         // [L][B]
    float tau_s, tau_H;
    int L;
};

// tau_base * (1 + lambda*[s > tau_s] + gamma*[H > tau_H]), in the association of the printed formula
__device__ __forceinline__ float tau_final_f32(float tau_base, float lambda, float gamma, float s, float H,
                                               float tau_s, float tau_H)
{
    const float is = s > tau_s ? 1.0f : 0.0f;
    const float ih = H > tau_H ? 1.0f : 0.0f;
    return tau_base * (1.0f + lambda * is + gamma * ih);
}

template <int ES>
__global__ void __launch_bounds__(SIG_THREADS)
k_signals(const char *__restrict__ logits, int V, const int32_t *__restrict__ tok,
          float *__restrict__ part /* [B][NB][4] */, int *__restrict__ counters,
          float *__restrict__ surprisal, float *__restrict__ entropy, const ThresholdTail th)
{
    __shared__ Lse s_w[SIG_THREADS / 64];
    __shared__ int s_last;
    const int b = blockIdx.y, nb = gridDim.x, tid = threadIdx.x;
    const char *row = logits + (size_t)b * V * ES;
    const int lo = blockIdx.x * SIG_CHUNK;
    const int hi = min(V, lo + SIG_CHUNK);

    Lse acc = lse_empty();
    for (int base = lo + tid; base < hi; base += SIG_THREADS * SIG_GROUP) {
        float z[SIG_GROUP];
        float gm = -INFINITY;
#pragma unroll
        for (int g = 0; g < SIG_GROUP; ++g) {
            const int v = base + g * SIG_THREADS;
            z[g] = v < hi ? load_logit<ES>(row, v) : -INFINITY;
            if (z[g] != z[g] || z[g] == INFINITY) acc.bad = 1;
            gm = fmaxf(gm, z[g]);
        }
        if (gm > acc.m) {                       // rescale once per group
            if (acc.Z > 0.0f) {
                const float dm = acc.m - gm, c = expf(dm);
                acc.T = c * (acc.T + dm * acc.Z);
                acc.Z = c * acc.Z;
            }
            acc.m = gm;
        }
#pragma unroll
        for (int g = 0; g < SIG_GROUP; ++g) {
            const float dz = z[g] - acc.m;
            const float e = expf(dz);
            if (e > 0.0f) {                      // -inf logits contribute nothing (0 log 0 := 0)
                acc.Z += e;
                acc.T += e * dz;
            }
        }
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        Lse other;
        other.m = __shfl_xor(acc.m, o);
        other.Z = __shfl_xor(acc.Z, o);
        other.T = __shfl_xor(acc.T, o);
        other.bad = __shfl_xor(acc.bad, o);
        // merge lower lane first so both partners compute the identical value
        acc = ((tid & o) == 0) ? lse_merge(acc, other) : lse_merge(other, acc);
    }
    if ((tid & 63) == 0) s_w[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) {
        Lse r = s_w[0];
        for (int w = 1; w < SIG_THREADS / 64; ++w) r = lse_merge(r, s_w[w]);
        // agent-scope (write-through) stores, one release at that scope, then the arrival count: the block
        // that folds the partials may run on another XCD
        float *dst = part + ((size_t)b * nb + blockIdx.x) * 4;
        __hip_atomic_store(dst + 0, r.m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(dst + 1, r.Z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(dst + 2, r.T, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(dst + 3, r.bad ? 1.0f : 0.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        const int prev = __hip_atomic_fetch_add(&counters[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == nb - 1);
        if (prev == nb - 1) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // the other blocks' partials
    }
    __syncthreads();
    if (s_last && tid < 64) {
        // last block of the row: lane l folds partials l, l + 64, ... in ascending order (all loads of the
        // wave in flight together), then the lanes merge by the same fixed butterfly as above
        Lse r = lse_empty();
        for (int q = tid; q < nb; q += 64) {
            const float *src = part + ((size_t)b * nb + q) * 4;
            Lse t;
            t.m = __hip_atomic_load(src + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            t.Z = __hip_atomic_load(src + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            t.T = __hip_atomic_load(src + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            t.bad = __hip_atomic_load(src + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0.0f;
            r = lse_merge(r, t);
        }
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            Lse other;
            other.m = __shfl_xor(r.m, o);
            other.Z = __shfl_xor(r.Z, o);
            other.T = __shfl_xor(r.T, o);
            other.bad = __shfl_xor(r.bad, o);
            r = ((tid & o) == 0) ? lse_merge(r, other) : lse_merge(other, r);
        }
        float H = 0.0f, s = 0.0f;
        if (tid == 0) {
            __hip_atomic_store(&counters[b], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
            if (r.bad || !(r.Z > 0.0f)) {
                H = NAN;
                s = NAN;
            } else {
                const float logZ = logf(r.Z);
                H = logZ - r.T / r.Z;
                const int t = tok[b];
                s = (t >= 0 && t < V) ? (r.m + logZ) - load_logit<ES>(row, t) : NAN;
            }
            entropy[b] = H;
            surprisal[b] = s;
        }
        if (th.L > 0) {                         // this row's thresholds for every layer, from the registers
            H = __shfl(H, 0);
            s = __shfl(s, 0);
            const int B = gridDim.y;
            for (int l = tid; l < th.L; l += 64)
                th.tau_final[(size_t)l * B + b] =
                    tau_final_f32(th.tau_base[l], th.lambda[l], th.gamma[l], s, H, th.tau_s, th.tau_H);
        }
    }
}

__global__ void __launch_bounds__(256)
k_threshold(const float *__restrict__ tau_base, const float *__restrict__ lambda,
            const float *__restrict__ gamma, int L, const float *__restrict__ s,
            const float *__restrict__ H, int B, float tau_s, float tau_H, float *__restrict__ out)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= L * B) return;
    const int l = idx / B, b = idx - l * B;
    out[idx] = tau_final_f32(tau_base[l], lambda[l], gamma[l], s[b], H[b], tau_s, tau_H);
}

}  // namespace

static int signals_blocks(int V) { return (V + SIG_CHUNK - 1) / SIG_CHUNK; }

size_t clada_ws_signals(int32_t B, int32_t V)
{
    if (B <= 0 || V <= 0) return 0;
    return align_up(sizeof(float) * 4 * (size_t)B * signals_blocks(V), 256);
}

// Argument checks shared by the three signal entry points (host only, before any HIP call).
static clada_status check_signals_args(clada_ctx *ctx, const void *logits, int32_t logits_dtype, int32_t B, int32_t V,
                                       const int32_t *token_ids, const float *surprisal, const float *entropy)
{
    if (!logits || !token_ids || !surprisal || !entropy)
        return clada_fail(ctx, CLADA_ERR_NULL, "logits, token_ids, surprisal or entropy is NULL");
    if (logits_dtype != CLADA_F32 && logits_dtype != CLADA_BF16)
        return clada_fail(ctx, CLADA_ERR_DTYPE, "unknown logits dtype %d", (int)logits_dtype);
    if (B < 1 || B > CLADA_MAX_BATCH) return clada_fail(ctx, CLADA_ERR_SHAPE, "B=%d outside [1,%d]", B, CLADA_MAX_BATCH);
    if (V < 1 || V > (1 << 24)) return clada_fail(ctx, CLADA_ERR_SHAPE, "V=%d outside [1,2^24]", V);
    if (((uintptr_t)logits & (dtype_size(logits_dtype) - 1)) != 0)
        return clada_fail(ctx, CLADA_ERR_ALIGN, "logits not aligned to their element size");
    return CLADA_OK;
}

static clada_status check_threshold_args(clada_ctx *ctx, const float *tau_base, const float *lambda, const float *gamma,
                                         int32_t L, int32_t B, float tau_s, float tau_H, const float *tau_final)
{
    if (!tau_base || !lambda || !gamma || !tau_final)
        return clada_fail(ctx, CLADA_ERR_NULL, "an array pointer is NULL");
    if (L < 1 || L > CLADA_MAX_LAYERS) return clada_fail(ctx, CLADA_ERR_SHAPE, "L=%d outside [1,%d]", L, CLADA_MAX_LAYERS);
    if (B < 1 || B > CLADA_MAX_BATCH) return clada_fail(ctx, CLADA_ERR_SHAPE, "B=%d outside [1,%d]", B, CLADA_MAX_BATCH);
    if (tau_s != tau_s || tau_H != tau_H) return clada_fail(ctx, CLADA_ERR_VALUE, "tau_s or tau_H is NaN");
    return CLADA_OK;
}

static hipError_t launch_signals(const void *logits, int32_t logits_dtype, int32_t B, int32_t V, const int32_t *token_ids,
                                 float *part, int *counters, float *surprisal, float *entropy, const ThresholdTail &th,
                                 hipStream_t st)
{
    const dim3 grid(signals_blocks(V), B);
    if (logits_dtype == CLADA_F32)
        hipLaunchKernelGGL(k_signals<4>, grid, dim3(SIG_THREADS), 0, st, (const char *)logits, V, token_ids,
                           part, counters, surprisal, entropy, th);
    else
        hipLaunchKernelGGL(k_signals<2>, grid, dim3(SIG_THREADS), 0, st, (const char *)logits, V, token_ids,
                           part, counters, surprisal, entropy, th);
    return hipGetLastError();
}

extern "C" clada_status clada_cognitive_signals(clada_ctx *ctx, const void *logits,
                                                int32_t logits_dtype, int32_t B, int32_t V,
                                                const int32_t *token_ids, float *surprisal,
                                                float *entropy, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    clada_status cs = check_signals_args(ctx, logits, logits_dtype, B, V, token_ids, surprisal, entropy);
    if (cs != CLADA_OK) return cs;
    const size_t need = CLADA_WS_HEADER + clada_ws_signals(B, V);
    if (ctx->ws_bytes < need)
        return clada_fail(ctx, CLADA_ERR_WORKSPACE, "workspace %zu < %zu bytes needed", ctx->ws_bytes, need);
    int *counters = reinterpret_cast<int *>(ctx->ws) + CTR_SIGNALS;
    float *part = reinterpret_cast<float *>(ctx->ws + CLADA_WS_HEADER);
    ThresholdTail th = {};
    CLADA_CHECK_HIP(ctx, launch_signals(logits, logits_dtype, B, V, token_ids, part, counters, surprisal, entropy, th,
                                        (hipStream_t)hip_stream));
    return CLADA_OK;
}

extern "C" clada_status clada_signals_threshold(clada_ctx *ctx, const void *logits, int32_t logits_dtype, int32_t B,
                                                int32_t V, const int32_t *token_ids, const float *tau_base,
                                                const float *lambda, const float *gamma, int32_t L, float tau_s,
                                                float tau_H, float *surprisal, float *entropy, float *tau_final,
                                                void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    clada_status cs = check_signals_args(ctx, logits, logits_dtype, B, V, token_ids, surprisal, entropy);
    if (cs != CLADA_OK) return cs;
    cs = check_threshold_args(ctx, tau_base, lambda, gamma, L, B, tau_s, tau_H, tau_final);
    if (cs != CLADA_OK) return cs;
    const size_t need = CLADA_WS_HEADER + clada_ws_signals(B, V);
    if (ctx->ws_bytes < need)
        return clada_fail(ctx, CLADA_ERR_WORKSPACE, "workspace %zu < %zu bytes needed", ctx->ws_bytes, need);
    int *counters = reinterpret_cast<int *>(ctx->ws) + CTR_SIGNALS;
    float *part = reinterpret_cast<float *>(ctx->ws + CLADA_WS_HEADER);
    const ThresholdTail th = {tau_base, lambda, gamma, tau_final, tau_s, tau_H, L};
    CLADA_CHECK_HIP(ctx, launch_signals(logits, logits_dtype, B, V, token_ids, part, counters, surprisal, entropy, th,
                                        (hipStream_t)hip_stream));
    return CLADA_OK;
}

extern "C" clada_status clada_threshold(clada_ctx *ctx, const float *tau_base, const float *lambda,
                                        const float *gamma, int32_t L, const float *surprisal,
                                        const float *entropy, int32_t B, float tau_s, float tau_H,
                                        float *tau_final, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    if (!surprisal || !entropy) return clada_fail(ctx, CLADA_ERR_NULL, "an array pointer is NULL");
    clada_status cs = check_threshold_args(ctx, tau_base, lambda, gamma, L, B, tau_s, tau_H, tau_final);
    if (cs != CLADA_OK) return cs;
    if (ctx->ws_bytes == 0) return clada_fail(ctx, CLADA_ERR_WORKSPACE, "context has no device");
    const int n = L * B;
    hipLaunchKernelGGL(k_threshold, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)hip_stream, tau_base,
                       lambda, gamma, L, surprisal, entropy, B, tau_s, tau_H, tau_final);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    return CLADA_OK;
}

// ---------------------------------------------------------------------------------------------------
// clada_cognitive_signals for callers that cannot allocate (see clada.h).  The block partials and the
// arrival counters, which the entry point above keeps in the context's workspace, live in this file-scope
// device array; every GPU the library runs on holds its own copy until the process ends.
//   bytes [0, 256)   : arrival counters, one int32 per row (self-resetting: the block that folds a row
//                      stores 0 again, and the array starts zeroed when the code object is loaded)
//   bytes [256, end) : partials [B][blocks][4] fp32
constexpr int STATIC_SIG_BLOCKS = CLADA_STATIC_SIGNALS_MAX_V / SIG_CHUNK;
constexpr size_t STATIC_SIG_BYTES = 256 + sizeof(float) * 4 * (size_t)CLADA_MAX_BATCH * STATIC_SIG_BLOCKS;
static_assert(CLADA_STATIC_SIGNALS_MAX_V % SIG_CHUNK == 0, "whole blocks");
static_assert(sizeof(int) * CLADA_MAX_BATCH <= 256, "counters fit their slot");
static __device__ __align__(256) unsigned char scratch[STATIC_SIG_BYTES];

// In host code `scratch` is only a handle for the runtime's symbol lookup, not a device address: the
// address of each device's copy is asked for once, with that device current, and kept here.
constexpr int STATIC_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static unsigned char *g_scratch_ptr[STATIC_MAX_DEVICES];

static hipError_t static_scratch_of_current_device(unsigned char **out, int *device_out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    *device_out = dev;
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<unsigned char *>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

extern "C" clada_status clada_cognitive_signals_static(clada_ctx *ctx, const void *logits, int32_t logits_dtype,
                                                       int32_t B, int32_t V, const int32_t *token_ids,
                                                       float *surprisal, float *entropy, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    clada_status cs = check_signals_args(ctx, logits, logits_dtype, B, V, token_ids, surprisal, entropy);
    if (cs != CLADA_OK) return cs;
    if (V > CLADA_STATIC_SIGNALS_MAX_V)
        return clada_fail(ctx, CLADA_ERR_SHAPE, "V=%d exceeds %d, the most the static scratch array holds partials for",
                          V, CLADA_STATIC_SIGNALS_MAX_V);
    unsigned char *base = nullptr;
    int dev = -1;
    const hipError_t e = static_scratch_of_current_device(&base, &dev);
    if (e != hipSuccess)
        return clada_fail(ctx, CLADA_ERR_HIP, "address of the static scratch array on device %d: %s", dev,
                          hipGetErrorString(e));
    int *counters = reinterpret_cast<int *>(base);
    float *part = reinterpret_cast<float *>(base + 256);
    ThresholdTail th = {};
    CLADA_CHECK_HIP(ctx, launch_signals(logits, logits_dtype, B, V, token_ids, part, counters, surprisal, entropy, th,
                                        (hipStream_t)hip_stream));
    return CLADA_OK;
}
