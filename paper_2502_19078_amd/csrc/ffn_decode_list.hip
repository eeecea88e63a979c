// Batch-1 sparse FFN over a caller-supplied neuron list (prefix-static masks): the sparse
// forward pass of the algorithm "CLADA Inference" (arXiv 2502.19078) when the mask does not
// depend on the token.  Only the listed neurons' gate, up and down rows are read, so the kernel
// is a pure stream over 3 * n * d * e bytes, split evenly: workgroup q takes list entries
// [q n / P, (q+1) n / P).  Eight neurons at a time, one per wave for the two input-projection
// rows (wave-wide dot products), all eight waves for the output-projection rows (each wave owns
// a 1 KiB column slice of the row, so the partial y needs no cross-wave fold).  With PIPE the
// next eight neurons' loads are issued before the current eight are consumed.
#include <type_traits>

#include "clada_internal.h"

namespace {

struct ListParams {
    const char *wg, *wu, *wd, *x;
    const int *idx, *n_list;
    float *partial;             // [P][d]
    int d, F;
    int gelu;                   // sigma = tanh-form GELU instead of SiLU
    const float *b_in;          // RELU: input bias [F] or nullptr
};

constexpr int LIST_MAXSEG = 1024;       // list entries per workgroup

// RELU: the non-gated family -- no W_up rows, h = max(0, W_in[j,:] . x + b_in[j]).
template <int ES, int NCH, int NW, bool PIPE, bool RELU = false>
__global__ void __launch_bounds__(NW * 64)
k_ffn_decode_list(const ListParams p)
{
    constexpr int VEC = 16 / ES;
    constexpr int ROWB = NCH * 1024;
    constexpr int SL = (NCH + NW - 1) / NW;
    __shared__ int s_rows[LIST_MAXSEG];
    __shared__ float s_h[2][NW];
    __shared__ __align__(16) char s_x[ROWB];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int blk = blockIdx.x, P = gridDim.x;
    const int n = min(max(p.n_list[0], 0), p.F);
    const int lo = (int)((long long)blk * n / P), hi = (int)((long long)(blk + 1) * n / P);
    const int cnt = min(hi - lo, LIST_MAXSEG);
    for (int i = tid; i < cnt; i += NW * 64) s_rows[i] = min(max(p.idx[lo + i], 0), p.F - 1);
    for (int i = tid; i < ROWB / 16; i += NW * 64)
        reinterpret_cast<u32x4 *>(s_x)[i] = reinterpret_cast<const u32x4 *>(p.x)[i];
    __syncthreads();

    const int loff = lane * 16;
    float acc[SL][VEC];
#pragma unroll
    for (int s = 0; s < SL; ++s)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[s][e] = 0.0f;

    // all loads of one group of NW neurons: this wave's neuron's gate and up rows, and this wave's
    // column slice of every neuron's down row
    auto issue = [&](u32x4 (&g)[NCH], u32x4 (&u)[NCH], u32x4 (&dn)[NW][SL], int base) {
        const size_t off = (size_t)s_rows[base + wave] * ROWB + loff;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            g[c] = ld_stream16(p.wg + off + c * 1024);
            if (!RELU) u[c] = ld_stream16(p.wu + off + c * 1024);
        }
#pragma unroll
        for (int e = 0; e < NW; ++e) {
            const char *row = p.wd + (size_t)s_rows[base + e] * ROWB + loff;
#pragma unroll
            for (int s = 0; s < SL; ++s) {
                const int c = wave + s * NW;
                if (c < NCH) dn[e][s] = ld_stream16(row + c * 1024);
                else dn[e][s] = u32x4{0u, 0u, 0u, 0u};
            }
        }
    };
    // h = sigma(gate . x) * (up . x) of this wave's neuron; x comes from LDS a chunk at a time
    auto neuron_h = [&](const u32x4 (&g)[NCH], const u32x4 (&u)[NCH], int j) {
        float sg = 0.0f, su = 0.0f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const u32x4 xv = *reinterpret_cast<const u32x4 *>(s_x + c * 1024 + loff);
            sg = dot16<ES>(g[c], xv, sg);
            if (!RELU) su = dot16<ES>(u[c], xv, su);
        }
        sg = wave_sum(sg);
        if (RELU) {
            if (p.b_in) sg += p.b_in[j];
            return sg > 0.0f ? sg : (sg != sg ? sg : 0.0f);
        }
        su = wave_sum(su);
        return gate_sigma_f32(sg, p.gelu) * su;
    };
    auto down_fma = [&](const u32x4 (&dn)[NW][SL], const float *hs, int nvalid) {
#pragma unroll
        for (int e = 0; e < NW; ++e) {
            const float h = e < nvalid ? hs[e] : 0.0f;
#pragma unroll
            for (int s = 0; s < SL; ++s) {
                float w[VEC];
                unpack_row16(dn[e][s], w);
#pragma unroll
                for (int k = 0; k < VEC; ++k) acc[s][k] = fmaf(h, w[k], acc[s][k]);
            }
        }
    };
    int par = 0;
    auto consume = [&](const u32x4 (&g)[NCH], const u32x4 (&u)[NCH], const u32x4 (&dn)[NW][SL], int base) {
        const float h = neuron_h(g, u, s_rows[base + wave]);
        if (lane == 0) s_h[par][wave] = h;
        __syncthreads();
        down_fma(dn, s_h[par], NW);
        par ^= 1;
    };

    const int nfull = cnt / NW, tail = cnt - nfull * NW;
    if (PIPE) {
        u32x4 ga[NCH], ua[NCH], da[NW][SL], gb[NCH], ub[NCH], db[NW][SL];
        if (nfull > 0) issue(ga, ua, da, 0);
        // every path has a fixed number of loads in flight, so the waits count exactly
        for (int c = 0; c < nfull; c += 2) {
            if (c + 1 < nfull) {
                issue(gb, ub, db, (c + 1) * NW);
                consume(ga, ua, da, c * NW);
                if (c + 2 < nfull) {
                    issue(ga, ua, da, (c + 2) * NW);
                    consume(gb, ub, db, (c + 1) * NW);
                } else {
                    consume(gb, ub, db, (c + 1) * NW);
                }
            } else {
                consume(ga, ua, da, c * NW);
            }
        }
    } else {
        for (int c = 0; c < nfull; ++c) {
            u32x4 g[NCH], u[NCH], dn[NW][SL];
            issue(g, u, dn, c * NW);
            consume(g, u, dn, c * NW);
        }
    }
    if (tail > 0) {                                   // ragged last group: fewer than NW neurons
        const int base = nfull * NW;
        u32x4 g[NCH], u[NCH], dn[NW][SL];
        float h = 0.0f;
#pragma unroll
        for (int e = 0; e < NW; ++e) {
            if (e < tail) {
                const char *row = p.wd + (size_t)s_rows[base + e] * ROWB + loff;
#pragma unroll
                for (int s = 0; s < SL; ++s) {
                    const int c = wave + s * NW;
                    if (c < NCH) dn[e][s] = ld_stream16(row + c * 1024);
                    else dn[e][s] = u32x4{0u, 0u, 0u, 0u};
                }
            } else {
#pragma unroll
                for (int s = 0; s < SL; ++s) dn[e][s] = u32x4{0u, 0u, 0u, 0u};
            }
        }
        if (wave < tail) {
            const size_t off = (size_t)s_rows[base + wave] * ROWB + loff;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                g[c] = ld_stream16(p.wg + off + c * 1024);
                if (!RELU) u[c] = ld_stream16(p.wu + off + c * 1024);
            }
            h = neuron_h(g, u, s_rows[base + wave]);
        }
        if (lane == 0) s_h[par][wave] = h;
        __syncthreads();
        down_fma(dn, s_h[par], tail);
    }

    float *dst = p.partial + (size_t)blk * p.d;
#pragma unroll
    for (int s = 0; s < SL; ++s) {
        const int c = wave + s * NW;
        if (c < NCH) {
#pragma unroll
            for (int k = 0; k < VEC; k += 4)
                *reinterpret_cast<float4 *>(dst + (c * 64 + lane) * VEC + k) =
                    make_float4(acc[s][k], acc[s][k + 1], acc[s][k + 2], acc[s][k + 3]);
        }
    }
}

template <int ES, int NCH, bool PIPE>
hipError_t launch_list(const ListParams &p, int P, hipStream_t st, bool relu)
{
    if (relu) hipLaunchKernelGGL((k_ffn_decode_list<ES, NCH, 8, PIPE, true>), dim3(P), dim3(512), 0, st, p);
    else      hipLaunchKernelGGL((k_ffn_decode_list<ES, NCH, 8, PIPE>), dim3(P), dim3(512), 0, st, p);
    return hipGetLastError();
}

}  // namespace

// Runs the batch-1 list kernel when the shape fits it (whole-KiB rows of 2, 8 or 10 KiB, at most
// LIST_MAXSEG entries per workgroup); *ran tells whether it did.  partial is [P][d] fp32; the
// caller launches the final reduction over *P_out partials.
hipError_t clada_decode_list_b1(clada_ctx *ctx, const clada_layer *layer, const void *x, const int32_t *idx,
                                const int32_t *n_active, float *partial, int *P_out, hipStream_t stream, bool *ran)
{
    *ran = false;
    const int d = layer->d, F = layer->d_ff, es = (int)dtype_size(layer->dtype);
    if ((d * es) % 1024 != 0) return hipSuccess;
    const int nch = d * es / 1024;
    const int P = ctx->num_cu < COOP_MAX_WGS ? ctx->num_cu : COOP_MAX_WGS;
    if (P < 1 || (F + P - 1) / P > LIST_MAXSEG) return hipSuccess;
    ListParams p;
    p.wg = (const char *)layer->w_gate; p.wu = (const char *)layer->w_up; p.wd = (const char *)layer->w_down;
    p.x = (const char *)x; p.idx = idx; p.n_list = n_active; p.partial = partial; p.d = d; p.F = F;
    p.gelu = layer->kind == CLADA_FFN_GEGLU ? 1 : 0;
    const bool relu = layer->kind == CLADA_FFN_RELU;
    p.b_in = relu ? layer->b_in : nullptr;
    hipError_t e;
    if (es == 2 && nch == 8) e = launch_list<2, 8, true>(p, P, stream, relu);
    else if (es == 2 && nch == 10) e = launch_list<2, 10, false>(p, P, stream, relu);
    else if (es == 2 && nch == 5) e = launch_list<2, 5, true>(p, P, stream, relu);
    else if (es == 2 && nch == 2) e = launch_list<2, 2, true>(p, P, stream, relu);
    else if (es == 4 && nch == 2) e = launch_list<4, 2, true>(p, P, stream, relu);
    else if (es == 4 && nch == 8) e = launch_list<4, 8, true>(p, P, stream, relu);
    else return hipSuccess;
    *P_out = P;
    *ran = true;
    return e;
}
