// Error-bounded base-threshold search (arXiv 2502.19078, section 3.2.2, base-threshold equation):
//     tau_base = max eps  s.t.  mean over validation tokens of CETT(x; eps) <= bound,
//     CETT(x; eps) = || sum_{j : |a_j(x)| < eps} h_j(x) W_down[j,:] ||_2 / || MLP(x) ||_2.
//
// The gate/up GEMM runs once (|a| pool and h stay in the workspace), the dense down projection
// gives the denominators, and every probe of eps is one masking pass over h plus one down
// projection whose epilogue reduces the output rows to sums of squares.  The search is a
// bisection on the bit pattern of the non-negative float eps (monotone in eps), with the bracket
// kept on the device: lo always satisfies the bound, hi never does, 31 probes resolve the float.
#include "clada_internal.h"

namespace {

struct CettState {
    unsigned int lo, hi, mid;     // float bit patterns; the probe in flight is `mid`
    float mean_lo, mean_mid;      // mean CETT at lo / at the last probe
};

// den[t] = || MLP(x_t) ||_2 from the per-column-tile sums of squares (ascending tile order);
// thread 0 of block 0 sets up the bracket, or the single probe of an evaluation call.
__global__ void __launch_bounds__(256)
k_cett_begin(CettState *st, const float *__restrict__ rowsq, int n_tn, int T, float *__restrict__ den,
             int search, float eps)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < T && rowsq) {                 // (the non-gated family's denominators come from k_cett_row_norm)
        float s = 0.0f;
        for (int i = 0; i < n_tn; ++i) s += rowsq[(size_t)i * T + t];
        den[t] = sqrtf(s);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        st->lo = 0u;                      // eps = 0 cuts nothing: CETT = 0
        st->hi = 0x7f800000u;             // eps = +inf cuts everything: CETT = 1 > bound
        st->mid = search ? (0x7f800000u >> 1) : __float_as_uint(eps);
        st->mean_lo = 0.0f;
        st->mean_mid = 0.0f;
    }
}

// den[t] = || y[t,:] ||_2 of a stored output (layer dtype): the denominators of the non-gated family, whose
// output carries the bias b_out that no neuron owns (the projection's own epilogue adds it to y; the row-norm
// epilogues do not know about it).  One wave per token: lane-strided sums of squares, then a fixed butterfly.
template <int ES>
__global__ void __launch_bounds__(256)
k_cett_row_norm(const char *__restrict__ y, int T, int d, float *__restrict__ den)
{
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (t >= T) return;
    const char *row = y + (size_t)t * d * ES;
    float s = 0.0f;
    for (int i = lane; i < d; i += 64) {
        const float v = ES == 4 ? reinterpret_cast<const float *>(row)[i]
                                : __uint_as_float((unsigned int)reinterpret_cast<const unsigned short *>(row)[i] << 16);
        s = fmaf(v, v, s);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) den[t] = sqrtf(s);
}

// hcut = h where |a| < eps (strict, NaN never cut), 0 elsewhere; eps = the probe in the state.
// One thread per 8 neurons when the rows allow 16-byte accesses, else per neuron.
template <int ES>
__global__ void __launch_bounds__(256)
k_cett_mask(const CettState *__restrict__ st, const float *__restrict__ pool, const char *__restrict__ h,
            char *__restrict__ hcut, int T, int F, int Fp)
{
    const float eps = __uint_as_float(st->mid);
    const size_t groups = (size_t)Fp / 8;
    const size_t total = (size_t)T * groups;
    for (size_t g = (size_t)blockIdx.x * 256 + threadIdx.x; g < total; g += (size_t)gridDim.x * 256) {
        const size_t t = g / groups;
        const int j0 = (int)(g % groups) * 8;
        const float *pr = pool + t * (size_t)F;
        const char *hr = h + (t * (size_t)Fp + j0) * ES;
        char *dr = hcut + (t * (size_t)Fp + j0) * ES;
        bool cut[8];
        if (F % 4 == 0 && j0 + 8 <= F) {
            const float4 p0 = *reinterpret_cast<const float4 *>(pr + j0);
            const float4 p1 = *reinterpret_cast<const float4 *>(pr + j0 + 4);
            cut[0] = p0.x < eps; cut[1] = p0.y < eps; cut[2] = p0.z < eps; cut[3] = p0.w < eps;
            cut[4] = p1.x < eps; cut[5] = p1.y < eps; cut[6] = p1.z < eps; cut[7] = p1.w < eps;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) cut[e] = (j0 + e < F) && (pr[j0 + e] < eps);
        }
        if (ES == 2) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(hr);
            u32x4 o;
            o.x = (cut[0] ? v.x & 0x0000ffffu : 0u) | (cut[1] ? v.x & 0xffff0000u : 0u);
            o.y = (cut[2] ? v.y & 0x0000ffffu : 0u) | (cut[3] ? v.y & 0xffff0000u : 0u);
            o.z = (cut[4] ? v.z & 0x0000ffffu : 0u) | (cut[5] ? v.z & 0xffff0000u : 0u);
            o.w = (cut[6] ? v.w & 0x0000ffffu : 0u) | (cut[7] ? v.w & 0xffff0000u : 0u);
            *reinterpret_cast<u32x4 *>(dr) = o;
        } else {
            const u32x4 v0 = *reinterpret_cast<const u32x4 *>(hr), v1 = *reinterpret_cast<const u32x4 *>(hr + 16);
            u32x4 o0, o1;
            o0.x = cut[0] ? v0.x : 0u; o0.y = cut[1] ? v0.y : 0u; o0.z = cut[2] ? v0.z : 0u; o0.w = cut[3] ? v0.w : 0u;
            o1.x = cut[4] ? v1.x : 0u; o1.y = cut[5] ? v1.y : 0u; o1.z = cut[6] ? v1.z : 0u; o1.w = cut[7] ? v1.w : 0u;
            *reinterpret_cast<u32x4 *>(dr) = o0;
            *reinterpret_cast<u32x4 *>(dr + 16) = o1;
        }
    }
}

// One workgroup: per-token CETT of the probe, their mean in a fixed order (thread i sums tokens
// i, i+1024, ...; then a tree over the threads), and the bisection step.
__global__ void __launch_bounds__(1024)
k_cett_update(CettState *st, const float *__restrict__ rowsq, int n_tn, int T, const float *__restrict__ den,
              float bound, int search, float *__restrict__ cett_out, float *__restrict__ mean_out)
{
    __shared__ float s_sum[1024];
    const int tid = threadIdx.x;
    float acc = 0.0f;
    for (int t = tid; t < T; t += 1024) {
        float s = 0.0f;
        for (int i = 0; i < n_tn; ++i) s += rowsq[(size_t)i * T + t];
        const float dn = den[t];
        const float c = dn > 0.0f ? sqrtf(s) / dn : 0.0f;       // a zero dense output has nothing to lose
        if (cett_out) cett_out[t] = c;
        acc += c;
    }
    s_sum[tid] = acc;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if (tid < w) s_sum[tid] += s_sum[tid + w];
        __syncthreads();
    }
    if (tid == 0) {
        const float mean = s_sum[0] / (float)T;
        st->mean_mid = mean;
        if (mean_out) *mean_out = mean;
        if (search) {
            unsigned int lo = st->lo, hi = st->hi;
            const unsigned int mid = st->mid;
            if (mean <= bound) { lo = mid; st->mean_lo = mean; }     // NaN fails the test: treated as over the bound
            else hi = mid;
            st->lo = lo;
            st->hi = hi;
            st->mid = lo + ((hi - lo) >> 1);
        }
    }
}

__global__ void k_cett_finish(const CettState *st, float *tau_out, float *mean_out)
{
    if (threadIdx.x == 0) {
        *tau_out = __uint_as_float(st->lo);
        if (mean_out) *mean_out = st->mean_lo;
    }
}

struct CettWs {
    float *part, *pool, *rowsq_den, *rowsq_num, *den, *splitk;
    char *h, *hcut, *ytmp;
    CettState *state;
};

CettWs carve(char *ws, int d, int F, int T)
{
    const size_t n_tm = (size_t)clada_prefix_token_tiles(T), n_tn = (size_t)clada_prefix_col_tiles(d);
    const size_t Fp = align_up((size_t)F, 64);
    CettWs w;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *p = ws + off; off += align_up(bytes, 256); return p; };
    w.part = reinterpret_cast<float *>(take(sizeof(float) * 4 * n_tm * F));
    w.pool = reinterpret_cast<float *>(take(sizeof(float) * (size_t)T * F));
    w.h = take((size_t)T * Fp * 4);
    w.hcut = take((size_t)T * Fp * 4);
    w.rowsq_den = reinterpret_cast<float *>(take(sizeof(float) * n_tn * T));
    w.rowsq_num = reinterpret_cast<float *>(take(sizeof(float) * n_tn * T));
    w.den = reinterpret_cast<float *>(take(sizeof(float) * (size_t)T));
    w.state = reinterpret_cast<CettState *>(take(sizeof(CettState)));
    w.ytmp = take((size_t)T * d * 4);
    const size_t sk = clada_ws_down_splitk(d, F, T);
    w.splitk = sk ? reinterpret_cast<float *>(take(sk)) : nullptr;
    return w;
}

clada_status check_common(clada_ctx *ctx, const clada_layer *layer, const void *x, int32_t T)
{
    if (!ctx) return CLADA_ERR_NULL;
    clada_status st = clada_check_layer(ctx, layer);
    if (st != CLADA_OK) return st;
    if (!x) return clada_fail(ctx, CLADA_ERR_NULL, "x_val is NULL");
    if (T < 1 || T > (1 << 20)) return clada_fail(ctx, CLADA_ERR_SHAPE, "T=%d outside [1,2^20]", T);
    if (!aligned16(x)) return clada_fail(ctx, CLADA_ERR_ALIGN, "x_val must be 16-byte aligned");
    const size_t need = CLADA_WS_HEADER + clada_ws_cett(layer->d, layer->d_ff, T);
    if (ctx->ws_bytes < need)
        return clada_fail(ctx, CLADA_ERR_WORKSPACE, "workspace %zu < %zu bytes needed", ctx->ws_bytes, need);
    return CLADA_OK;
}

// Gate/up GEMM, dense down projection for the denominators, bracket / probe set-up.
clada_status begin(clada_ctx *ctx, const clada_layer *layer, const void *x, int T, const CettWs &w, int search,
                   float eps, hipStream_t stream)
{
    const int n_tn = clada_prefix_col_tiles(layer->d);
    CLADA_CHECK_HIP(ctx, clada_prefix_gateup(layer, x, T, w.part, w.pool, w.h, ctx->opt_prefix_tile, stream));
    const float *rowsq_den = w.rowsq_den;
    if (layer->kind == CLADA_FFN_RELU) {
        // || sum_j a_j W_out[j,:] + b_out ||: through the stored output, which carries the bias
        CLADA_CHECK_HIP(ctx, clada_prefix_down(layer, w.h, T, w.ytmp, nullptr, w.splitk, ctx->opt_prefix_tile, stream));
        if (layer->dtype == CLADA_BF16)
            hipLaunchKernelGGL(k_cett_row_norm<2>, dim3((T + 3) / 4), dim3(256), 0, stream, w.ytmp, T, layer->d, w.den);
        else
            hipLaunchKernelGGL(k_cett_row_norm<4>, dim3((T + 3) / 4), dim3(256), 0, stream, w.ytmp, T, layer->d, w.den);
        CLADA_CHECK_HIP(ctx, hipGetLastError());
        rowsq_den = nullptr;
    } else {
        CLADA_CHECK_HIP(ctx, clada_prefix_down(layer, w.h, T, nullptr, w.rowsq_den, w.splitk, ctx->opt_prefix_tile, stream));
    }
    hipLaunchKernelGGL(k_cett_begin, dim3((T + 255) / 256), dim3(256), 0, stream, w.state, rowsq_den, n_tn, T,
                       w.den, search, eps);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    return CLADA_OK;
}

// One probe: mask h at the state's eps, project, reduce, (bisect).
clada_status probe(clada_ctx *ctx, const clada_layer *layer, int T, const CettWs &w, float bound, int search,
                   float *cett_out, float *mean_out, hipStream_t stream)
{
    const int d = layer->d, F = layer->d_ff, n_tn = clada_prefix_col_tiles(d);
    const int Fp = (int)align_up((size_t)F, 64);
    const size_t groups = (size_t)T * (Fp / 8);
    const int grid = (int)((groups + 255) / 256 < 4096 ? (groups + 255) / 256 : 4096);
    if (layer->dtype == CLADA_BF16)
        hipLaunchKernelGGL(k_cett_mask<2>, dim3(grid), dim3(256), 0, stream, w.state, w.pool, w.h, w.hcut, T, F, Fp);
    else
        hipLaunchKernelGGL(k_cett_mask<4>, dim3(grid), dim3(256), 0, stream, w.state, w.pool, w.h, w.hcut, T, F, Fp);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    CLADA_CHECK_HIP(ctx, clada_prefix_down(layer, w.hcut, T, nullptr, w.rowsq_num, w.splitk, ctx->opt_prefix_tile, stream));
    hipLaunchKernelGGL(k_cett_update, dim3(1), dim3(1024), 0, stream, w.state, w.rowsq_num, n_tn, T, w.den, bound,
                       search, cett_out, mean_out);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    return CLADA_OK;
}

}  // namespace

size_t clada_ws_cett(int32_t d, int32_t d_ff, int32_t T)
{
    if (T <= 0) return 0;
    const size_t n_tm = (size_t)clada_prefix_token_tiles(T), n_tn = (size_t)clada_prefix_col_tiles(d);
    const size_t Fp = align_up((size_t)d_ff, 64);
    return align_up(sizeof(float) * 4 * n_tm * d_ff, 256) + align_up(sizeof(float) * (size_t)T * d_ff, 256) +
           2 * align_up((size_t)T * Fp * 4, 256) + 2 * align_up(sizeof(float) * n_tn * T, 256) +
           align_up(sizeof(float) * (size_t)T, 256) + 256 + align_up((size_t)T * d * 4, 256) +
           clada_ws_down_splitk(d, d_ff, T);
}

extern "C" clada_status clada_cett_eval(clada_ctx *ctx, const clada_layer *layer, const void *x_val, int32_t T,
                                        float eps, float *cett_out, float *mean_out, void *hip_stream)
{
    clada_status st = check_common(ctx, layer, x_val, T);
    if (st != CLADA_OK) return st;
    if (!cett_out && !mean_out) return clada_fail(ctx, CLADA_ERR_NULL, "cett_out and mean_out are both NULL");
    if (eps != eps) return clada_fail(ctx, CLADA_ERR_VALUE, "eps is NaN");
    hipStream_t stream = (hipStream_t)hip_stream;
    const CettWs w = carve(ctx->ws + CLADA_WS_HEADER, layer->d, layer->d_ff, T);
    st = begin(ctx, layer, x_val, T, w, 0, eps, stream);
    if (st != CLADA_OK) return st;
    return probe(ctx, layer, T, w, 0.0f, 0, cett_out, mean_out, stream);
}

extern "C" clada_status clada_threshold_search_cett(clada_ctx *ctx, const clada_layer *layer, const void *x_val,
                                                    int32_t T, float bound, int32_t n_probes, float *tau_base_out,
                                                    float *mean_cett_out, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    if (!tau_base_out) return clada_fail(ctx, CLADA_ERR_NULL, "tau_base_out is NULL");
    if (!(bound >= 0.0f && bound < 1.0f)) return clada_fail(ctx, CLADA_ERR_VALUE, "bound=%g outside [0,1)", (double)bound);
    if (n_probes < 1 || n_probes > 31) return clada_fail(ctx, CLADA_ERR_VALUE, "n_probes=%d outside [1,31]", n_probes);
    clada_status st = check_common(ctx, layer, x_val, T);
    if (st != CLADA_OK) return st;
    hipStream_t stream = (hipStream_t)hip_stream;
    const CettWs w = carve(ctx->ws + CLADA_WS_HEADER, layer->d, layer->d_ff, T);
    st = begin(ctx, layer, x_val, T, w, 1, 0.0f, stream);
    if (st != CLADA_OK) return st;
    for (int it = 0; it < n_probes; ++it) {
        st = probe(ctx, layer, T, w, bound, 1, nullptr, nullptr, stream);
        if (st != CLADA_OK) return st;
    }
    hipLaunchKernelGGL(k_cett_finish, dim3(1), dim3(64), 0, stream, w.state, tau_base_out, mean_cett_out);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    return CLADA_OK;
}
