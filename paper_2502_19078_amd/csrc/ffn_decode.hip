// Decode-time thresholded sparse SwiGLU FFN for one layer (algorithm "CLADA
// Inference", generation phase) and its dense twin, for gfx950.
//
// Work split.  Workgroup p of P owns the neurons j = p, p+P, p+2P, ... so that at
// any moment the chip streams a contiguous window of weight rows (all HBM
// channels busy).  Inside a workgroup every wavefront handles whole rows:
//   gate phase   : 16-byte loads of W_gate[j,:] (one row = d*elem bytes,
//                  contiguous), fp32 dot with x held in registers, DPP wave sum,
//                  a = SiLU(g), keep = |a| >= tau   (fp32 compare)
//   compaction   : wave 0 ballots the keep flags of the workgroup's neurons and
//                  prefix-sums them into an ascending list in LDS
//   up/down phase: kept neurons are dealt round-robin to the waves; a wave loads
//                  W_up[j,:] and W_down[j,:] together (the down loads do not
//                  depend on the dot), h = a * (W_up[j,:].x), acc += h*W_down[j,:]
//   reduction    : waves fold their fp32 accumulators through LDS in a fixed
//                  tree; the workgroup writes one partial y; a second kernel
//                  adds the P partials in fixed order and rounds once to the
//                  output dtype.  No atomics on floating point anywhere, so
//                  results are bit-reproducible.
#include "clada_internal.h"

namespace {

struct DecodeParams {
    const char *wg, *wu, *wd;   // [F][d] neuron-major
    const char *x;              // [B][d]
    const float *tau;           // [B] (unused when DENSE)
    float *partial;             // [P][B][d]
    unsigned char *keep;        // [B][F] or nullptr
    int d, F, ni_max;
};

__device__ __forceinline__ u32x4 ld_stream16(const char *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

// ES = element size (2: bf16, 4: fp32); NCH = 16-byte chunks per lane per row;
// NW = waves per workgroup; GB / UB = rows in flight per wave in the gate /
// up-down phase.
template <int ES, int NCH, int NW, int GB, int UB, bool DENSE>
__global__ void __launch_bounds__(NW * 64)
k_ffn_decode(const DecodeParams p)
{
    constexpr int VEC = 16 / ES;
    extern __shared__ __align__(16) unsigned char smem[];
    float *s_a = reinterpret_cast<float *>(smem);
    int *s_flag = reinterpret_cast<int *>(s_a + p.ni_max);
    int *s_list = s_flag + p.ni_max;
    int *s_cnt = s_list + p.ni_max;
    float *s_red = reinterpret_cast<float *>(smem + ((sizeof(int) * (3 * (size_t)p.ni_max + 4) + 15) & ~(size_t)15));

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int blk = blockIdx.x, P = gridDim.x, b = blockIdx.y;
    const int d = p.d, F = p.F;
    const size_t rowbytes = (size_t)d * ES;
    const int ni = blk < F ? (F - blk + P - 1) / P : 0;

    bool ok[NCH];
    int coff[NCH];
    float xr[NCH][VEC];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = (c * 64 + lane) * VEC;
        ok[c] = col < d;
        coff[c] = col * ES;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (ok[c]) v = *reinterpret_cast<const u32x4 *>(p.x + (size_t)b * rowbytes + coff[c]);
        unpack_row16(v, xr[c]);
    }
    const float tau = DENSE ? 0.0f : p.tau[b];

    // ---------------------------------------------------------------- gate phase
    for (int i0 = wave * GB; i0 < ni; i0 += NW * GB) {
        u32x4 buf[GB][NCH];
#pragma unroll
        for (int r = 0; r < GB; ++r) {
            const bool rv = i0 + r < ni;
            const char *row = p.wg + (size_t)(blk + (size_t)P * (rv ? i0 + r : i0)) * rowbytes;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (rv && ok[c]) v = ld_stream16(row + coff[c]);
                buf[r][c] = v;
            }
        }
#pragma unroll
        for (int r = 0; r < GB; ++r) {
            float s = 0.0f;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                float w[VEC];
                unpack_row16(buf[r][c], w);
#pragma unroll
                for (int e = 0; e < VEC; ++e) s = fmaf(w[e], xr[c][e], s);
            }
            s = wave_sum(s);
            const float a = silu_f32(s);
            const bool keep = DENSE ? true : (fabsf(a) >= tau);
            const int i = i0 + r;
            if (lane == 0 && i < ni) {
                s_a[i] = a;
                s_flag[i] = keep ? 1 : 0;
                if (p.keep) p.keep[(size_t)b * F + blk + (size_t)P * i] = keep ? 1 : 0;
            }
        }
    }
    __syncthreads();

    // -------------------------------------- compaction: ballot + popcount prefix sum
    if (wave == 0) {
        int cnt = 0;
        for (int base = 0; base < ni; base += 64) {
            const int i = base + lane;
            const bool k = i < ni && s_flag[i] != 0;
            const unsigned long long bal = __ballot(k);
            if (k) s_list[cnt + __popcll(bal & ((1ull << lane) - 1ull))] = i;
            cnt += __popcll(bal);
        }
        if (lane == 0) *s_cnt = cnt;
    }
    __syncthreads();
    const int cnt = *s_cnt;

    // ------------------------------------------------------------- up/down phase
    float acc[NCH][VEC];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[c][e] = 0.0f;

    for (int t0 = wave; t0 < cnt; t0 += NW * UB) {
        u32x4 ub[UB][NCH], db[UB][NCH];
        float av[UB];
#pragma unroll
        for (int r = 0; r < UB; ++r) {
            const int t = t0 + r * NW;
            const bool rv = t < cnt;
            const int i = rv ? s_list[t] : 0;
            av[r] = rv ? s_a[i] : 0.0f;
            const size_t off = (size_t)(blk + (size_t)P * i) * rowbytes;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                u32x4 u = {0u, 0u, 0u, 0u}, w = {0u, 0u, 0u, 0u};
                if (rv && ok[c]) {
                    u = ld_stream16(p.wu + off + coff[c]);
                    w = ld_stream16(p.wd + off + coff[c]);
                }
                ub[r][c] = u;
                db[r][c] = w;
            }
        }
#pragma unroll
        for (int r = 0; r < UB; ++r) {
            float s = 0.0f;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                float w[VEC];
                unpack_row16(ub[r][c], w);
#pragma unroll
                for (int e = 0; e < VEC; ++e) s = fmaf(w[e], xr[c][e], s);
            }
            const float h = av[r] * wave_sum(s);
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                float w[VEC];
                unpack_row16(db[r][c], w);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[c][e] = fmaf(h, w[e], acc[c][e]);
            }
        }
    }

    // ------------------------------------ fixed-order fold of the waves' accumulators
#pragma unroll
    for (int s = NW / 2; s >= 1; s >>= 1) {
        if (wave >= s && wave < 2 * s) {
            float *dst = s_red + (size_t)(wave - s) * (NCH * 64 * VEC);
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int e = 0; e < VEC; e += 4)
                    *reinterpret_cast<float4 *>(dst + (c * 64 + lane) * VEC + e) =
                        make_float4(acc[c][e], acc[c][e + 1], acc[c][e + 2], acc[c][e + 3]);
        }
        __syncthreads();
        if (wave < s) {
            const float *src = s_red + (size_t)wave * (NCH * 64 * VEC);
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int e = 0; e < VEC; e += 4) {
                    const float4 v = *reinterpret_cast<const float4 *>(src + (c * 64 + lane) * VEC + e);
                    acc[c][e] += v.x; acc[c][e + 1] += v.y; acc[c][e + 2] += v.z; acc[c][e + 3] += v.w;
                }
        }
        __syncthreads();
    }
    if (wave == 0) {
        float *dst = p.partial + ((size_t)blk * gridDim.y + b) * d;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
            if (ok[c]) {
#pragma unroll
                for (int e = 0; e < VEC; e += 4)
                    *reinterpret_cast<float4 *>(dst + (c * 64 + lane) * VEC + e) =
                        make_float4(acc[c][e], acc[c][e + 1], acc[c][e + 2], acc[c][e + 3]);
            }
    }
}

// y[b][col] = sum_p partial[p][b][col], p ascending within each of 16 strided
// slices, slices folded by a fixed tree; one rounding to the output dtype.
template <int ES>
__global__ void __launch_bounds__(256)
k_ffn_finalize(const float *__restrict__ partial, int P, int d, char *__restrict__ y)
{
    __shared__ float4 s_sum[16][16];
    const int cg = threadIdx.x & 15, sl = threadIdx.x >> 4;
    const int col = blockIdx.x * 64 + cg * 4;
    const int b = blockIdx.y, B = gridDim.y;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (col < d)
        for (int q = sl; q < P; q += 16) {
            const float4 v = *reinterpret_cast<const float4 *>(partial + ((size_t)q * B + b) * d + col);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
    s_sum[sl][cg] = s;
    __syncthreads();
#pragma unroll
    for (int h = 8; h >= 1; h >>= 1) {
        if (sl < h) {
            const float4 v = s_sum[sl + h][cg];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
            s_sum[sl][cg] = s;
        }
        __syncthreads();
    }
    if (sl == 0 && col < d) {
        if (ES == 4) {
            *reinterpret_cast<float4 *>(y + ((size_t)b * d + col) * 4) = s;
        } else {
            uint2 o;
            o.x = f32_to_bf16_bits(s.x) | (f32_to_bf16_bits(s.y) << 16);
            o.y = f32_to_bf16_bits(s.z) | (f32_to_bf16_bits(s.w) << 16);
            *reinterpret_cast<uint2 *>(y + ((size_t)b * d + col) * 2) = o;
        }
    }
}

// Ascending union index list, counts and per-token bit masks from the keep
// flags [B][F].  One workgroup of 1024 threads; all integer work.
__global__ void __launch_bounds__(1024)
k_ffn_lists(const unsigned char *__restrict__ keep, int B, int F, int32_t *__restrict__ active_idx,
            int32_t *__restrict__ n_active, uint32_t *__restrict__ mask_bits)
{
    __shared__ int s_wave_cnt[16];
    __shared__ int s_tok_cnt[CLADA_MAX_BATCH];
    __shared__ int s_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int words = (F + 31) / 32;
    if (tid < CLADA_MAX_BATCH) s_tok_cnt[tid] = 0;
    if (tid == 0) s_base = 0;
    __syncthreads();
    for (int base = 0; base < F; base += 1024) {
        const int j = base + tid;
        bool any = false;
        for (int b = 0; b < B; ++b) {
            const bool k = j < F && keep[(size_t)b * F + j] != 0;
            any |= k;
            const unsigned long long bal = __ballot(k);
            if (lane == 0) {
                if (bal) atomicAdd(&s_tok_cnt[b], __popcll(bal));
                if (mask_bits) {
                    const int w0 = (base + wave * 64) >> 5;
                    if (w0 < words) mask_bits[(size_t)b * words + w0] = (uint32_t)bal;
                    if (w0 + 1 < words) mask_bits[(size_t)b * words + w0 + 1] = (uint32_t)(bal >> 32);
                }
            }
        }
        const unsigned long long ubal = __ballot(any);
        if (lane == 0) s_wave_cnt[wave] = __popcll(ubal);
        __syncthreads();
        int off = s_base;
        for (int w = 0; w < wave; ++w) off += s_wave_cnt[w];
        if (any && active_idx) active_idx[off + __popcll(ubal & ((1ull << lane) - 1ull))] = j;
        __syncthreads();
        if (tid == 0) {
            int t = s_base;
            for (int w = 0; w < 16; ++w) t += s_wave_cnt[w];
            s_base = t;
        }
        __syncthreads();
    }
    if (n_active) {
        if (tid == 0) n_active[0] = s_base;
        if (tid < B) n_active[1 + tid] = s_tok_cnt[tid];
    }
}

template <int ES, int NCH, int NW, int GB, int UB>
hipError_t launch_decode(const DecodeParams &p, int P, int B, bool dense, hipStream_t st)
{
    constexpr int VEC = 16 / ES;
    const size_t lds = align_up(sizeof(int) * (3 * (size_t)p.ni_max + 4), 16) +
                       sizeof(float) * (size_t)(NW / 2) * NCH * 64 * VEC;
    auto kern = dense ? k_ffn_decode<ES, NCH, NW, GB, UB, true> : k_ffn_decode<ES, NCH, NW, GB, UB, false>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(P, B), dim3(NW * 64), lds, st, p);
    return hipGetLastError();
}

clada_status run_decode(clada_ctx *ctx, const clada_layer *layer, const void *x, int32_t B,
                        const float *tau, void *y, int32_t *active_idx, int32_t *n_active,
                        uint32_t *mask_bits, bool dense, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    clada_status st = clada_check_layer(ctx, layer);
    if (st != CLADA_OK) return st;
    if (!x || !y || (!dense && !tau)) return clada_fail(ctx, CLADA_ERR_NULL, "x, y or tau_final is NULL");
    if (B < 1 || B > CLADA_MAX_BATCH) return clada_fail(ctx, CLADA_ERR_SHAPE, "B=%d outside [1,%d]", B, CLADA_MAX_BATCH);
    if (!aligned16(x) || !aligned16(y)) return clada_fail(ctx, CLADA_ERR_ALIGN, "x and y must be 16-byte aligned");
    const int d = layer->d, F = layer->d_ff;
    const size_t need = CLADA_WS_HEADER + clada_ws_decode(d, F, B);
    if (ctx->ws_bytes < need)
        return clada_fail(ctx, CLADA_ERR_WORKSPACE, "workspace %zu < %zu bytes needed", ctx->ws_bytes, need);

    const int es = (int)dtype_size(layer->dtype);
    const bool lists = active_idx || n_active || mask_bits;
    int P = ctx->num_cu * ctx->opt_decode_wgs_per_cu;
    if (P > F) P = F;
    if (P > CLADA_MAX_DECODE_WGS) P = CLADA_MAX_DECODE_WGS;
    char *ws = ctx->ws + CLADA_WS_HEADER;
    DecodeParams p;
    p.wg = (const char *)layer->w_gate; p.wu = (const char *)layer->w_up; p.wd = (const char *)layer->w_down;
    p.x = (const char *)x; p.tau = tau;
    p.partial = reinterpret_cast<float *>(ws);
    p.keep = lists ? reinterpret_cast<unsigned char *>(ws + align_up(sizeof(float) * (size_t)CLADA_MAX_DECODE_WGS * B * d, 256)) : nullptr;
    p.d = d; p.F = F; p.ni_max = (F + P - 1) / P;
    hipStream_t stream = (hipStream_t)hip_stream;

    const int nch = (d * es + 1023) / 1024;
    hipError_t e = hipErrorInvalidValue;
#define CLADA_DECODE_CASE(ES_, NCH_, NW_, GB_, UB_)                                        \
    if (es == ES_ && nch <= NCH_ && e == hipErrorInvalidValue)                             \
        e = launch_decode<ES_, NCH_, NW_, GB_, UB_>(p, P, B, dense, stream);
    CLADA_DECODE_CASE(2, 1, 8, 2, 2)
    CLADA_DECODE_CASE(2, 2, 8, 2, 2)
    CLADA_DECODE_CASE(2, 4, 8, 2, 2)
    CLADA_DECODE_CASE(2, 8, 8, 2, 1)
    CLADA_DECODE_CASE(2, 10, 8, 2, 1)
    CLADA_DECODE_CASE(2, 16, 8, 1, 1)
    CLADA_DECODE_CASE(4, 1, 8, 2, 2)
    CLADA_DECODE_CASE(4, 2, 8, 2, 2)
    CLADA_DECODE_CASE(4, 4, 8, 2, 2)
    CLADA_DECODE_CASE(4, 8, 8, 2, 1)
    CLADA_DECODE_CASE(4, 16, 8, 1, 1)
#undef CLADA_DECODE_CASE
    CLADA_CHECK_HIP(ctx, e);

    dim3 fgrid((d + 63) / 64, B);
    if (es == 4) hipLaunchKernelGGL(k_ffn_finalize<4>, fgrid, dim3(256), 0, stream, p.partial, P, d, (char *)y);
    else         hipLaunchKernelGGL(k_ffn_finalize<2>, fgrid, dim3(256), 0, stream, p.partial, P, d, (char *)y);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    if (lists) {
        hipLaunchKernelGGL(k_ffn_lists, dim3(1), dim3(1024), 0, stream, p.keep, B, F, active_idx, n_active, mask_bits);
        CLADA_CHECK_HIP(ctx, hipGetLastError());
    }
    return CLADA_OK;
}

}  // namespace

size_t clada_ws_decode(int32_t d, int32_t d_ff, int32_t B)
{
    if (B <= 0) return 0;
    return align_up(sizeof(float) * (size_t)CLADA_MAX_DECODE_WGS * B * d, 256) + align_up((size_t)B * d_ff, 256);
}

extern "C" clada_status clada_sparse_ffn_decode(clada_ctx *ctx, const clada_layer *layer, const void *x,
                                                int32_t B, const float *tau_final, void *y,
                                                int32_t *active_idx, int32_t *n_active,
                                                uint32_t *mask_bits, void *hip_stream)
{
    return run_decode(ctx, layer, x, B, tau_final, y, active_idx, n_active, mask_bits, false, hip_stream);
}

extern "C" clada_status clada_dense_ffn_decode(clada_ctx *ctx, const clada_layer *layer, const void *x,
                                               int32_t B, void *y, void *hip_stream)
{
    return run_decode(ctx, layer, x, B, nullptr, y, nullptr, nullptr, nullptr, true, hip_stream);
}
