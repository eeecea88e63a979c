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
#include <type_traits>

#include <hip/hip_ext.h>

#include "clada_internal.h"

namespace {

// The partial-output region at the start of the decode scratch: [P][B][d] fp32 for up to CLADA_MAX_DECODE_WGS
// workgroups, and at least four buffers of [COOP_MAX_WGS][d] for the whole-stack calls at B = 1 (one per lane, two
// for chained launches, three for the persistent kernel).
size_t ws_partial_bytes(int B, int d)
{
    size_t rows = (size_t)CLADA_MAX_DECODE_WGS * B;
    if (rows < 4 * (size_t)COOP_MAX_WGS) rows = 4 * (size_t)COOP_MAX_WGS;
    return align_up(sizeof(float) * rows * d, 256);
}

struct DecodeParams {
    const char *wg, *wu, *wd;   // [F][d] neuron-major
    const char *x;              // [B][d]
    const float *tau;           // [B] (unused when DENSE)
    float *partial;             // [P][B][d]
    unsigned char *keep;        // [B][F] or nullptr
    const int *idx;             // LIST: neuron indices to run (ascending), device
    const int *n_list;          // LIST: their count, device
    const float *b_in;          // RELU: input bias [F] or nullptr
    int d, F, ni_max;
    int gelu;                   // gated family: sigma = tanh-form GELU instead of SiLU
};

// Activation of the FFN families: sigma(g) (SiLU or tanh-form GELU) for the gated FFN; for the
// non-gated one max(0, g + bias) (a NaN pre-activation stays NaN).
template <bool RELU>
__device__ __forceinline__ float ffn_act(float g, const float *b_in, size_t j, int gelu)
{
    if (!RELU) return gate_sigma_f32(g, gelu);
    if (b_in) g += b_in[j];
    return g > 0.0f ? g : (g != g ? g : 0.0f);
}


// ES = element size (2: bf16, 4: fp32); NCH = 16-byte chunks per lane per row;
// NW = waves per workgroup; GB / UB = rows in flight per wave in the gate /
// up-down phase.  LIST (with DENSE): the neurons are entries blk, blk+P, ... of a caller-supplied
// index list instead of rows blk, blk+P, ... of the matrices; every listed neuron is kept.
// RELU: the non-gated family (no W_up pass, h = a).
template <int ES, int NCH, int NW, int GB, int UB, bool DENSE, bool LIST = false, bool RELU = false>
__global__ void __launch_bounds__(NW * 64)
k_ffn_decode(const DecodeParams p)
{
    static_assert(!LIST || DENSE, "a list run keeps every listed neuron");
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
    int n_src = F;
    if (LIST) n_src = min(max(p.n_list[0], 0), F);
    const int ni = blk < n_src ? (n_src - blk + P - 1) / P : 0;
    auto neuron = [&](int i) -> size_t {
        if (LIST) return (size_t)min(max(p.idx[blk + (size_t)P * i], 0), F - 1);
        return blk + (size_t)P * i;
    };

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
            const char *row = p.wg + neuron(rv ? i0 + r : i0) * rowbytes;
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
            const int i = i0 + r;
            const float a = ffn_act<RELU>(s, p.b_in, neuron(i < ni ? i : i0), p.gelu);
            const bool keep = DENSE ? true : (fabsf(a) >= tau);
            if (lane == 0 && i < ni) {
                s_a[i] = a;
                s_flag[i] = keep ? 1 : 0;
                if (p.keep) p.keep[(size_t)b * F + neuron(i)] = keep ? 1 : 0;
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
            const size_t off = neuron(i) * rowbytes;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                u32x4 u = {0u, 0u, 0u, 0u}, w = {0u, 0u, 0u, 0u};
                if (rv && ok[c]) {
                    if (!RELU) u = ld_stream16(p.wu + off + coff[c]);
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
            const float h = RELU ? av[r] : av[r] * wave_sum(s);
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

// y[b][col] = sum_p partial[p][b][col].  A workgroup owns 4*CG columns; thread (slice, colgroup)
// adds the partials p = slice, slice+SL, ... (U loads in flight at a time), the SL slices are
// folded by a fixed tree; one rounding to the output dtype.
template <int ES, int CG, int SL, int U>
__global__ void __launch_bounds__(CG * SL)
k_ffn_finalize(const float *__restrict__ partial, int P, int d, char *__restrict__ y, unsigned int *epoch,
               const float *__restrict__ bias, const int *__restrict__ fault)
{
    if (epoch && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *epoch += 1u;   // cooperative call counter
    __shared__ float4 s_sum[SL][CG];
    const int cg = threadIdx.x % CG, sl = threadIdx.x / CG;
    const int col = blockIdx.x * (4 * CG) + cg * 4;
    const int b = blockIdx.y, B = gridDim.y;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (col < d) {
        const float *base = partial + (size_t)b * d + col;
        const size_t pstride = (size_t)B * d;
        int q = sl;
        for (; q + (U - 1) * SL < P; q += U * SL) {
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = *reinterpret_cast<const float4 *>(base + (size_t)(q + u * SL) * pstride);
#pragma unroll
            for (int u = 0; u < U; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
        }
        for (; q < P; q += SL) {
            const float4 v = *reinterpret_cast<const float4 *>(base + (size_t)q * pstride);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
    }
    s_sum[sl][cg] = s;
    __syncthreads();
#pragma unroll
    for (int h = SL / 2; h >= 1; h >>= 1) {
        if (sl < h) {
            const float4 v = s_sum[sl + h][cg];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
            s_sum[sl][cg] = s;
        }
        __syncthreads();
    }
    if (sl == 0 && col < d) {
        if (fault && *fault) s.x = s.y = s.z = s.w = __int_as_float(0x7fc00000);   // a balanced call gave up: no silent wrong sums
        if (bias) {                                     // output bias of the non-gated family
            const float4 bv = *reinterpret_cast<const float4 *>(bias + col);
            s.x += bv.x; s.y += bv.y; s.z += bv.z; s.w += bv.w;
        }
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

template <int ES, int CG, int SL, int U>
void launch_finalize_shape(const float *partial, int P, int B, int d, char *y, unsigned int *epoch, hipStream_t stream,
                           hipEvent_t ev_start, hipEvent_t ev_stop, const float *bias, const int *fault)
{
    const dim3 grid((d + 4 * CG - 1) / (4 * CG), B);
    auto kern = k_ffn_finalize<ES, CG, SL, U>;
    if (ev_start) hipExtLaunchKernelGGL(kern, grid, dim3(CG * SL), 0, stream, ev_start, ev_stop, 0, partial, P, d, y, epoch, bias, fault);
    else hipLaunchKernelGGL(kern, grid, dim3(CG * SL), 0, stream, partial, P, d, y, epoch, bias, fault);
}

void launch_finalize(int es, const float *partial, int P, int B, int d, char *y, unsigned int *epoch, hipStream_t stream,
                     hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr, const float *bias = nullptr,
                     const int *fault = nullptr)
{
    // 8 column groups x 32 slices, 8 loads in flight per thread.  The kernel is one dependent round trip
    // through memory plus its launch, about 4 us whatever its shape: 64 to 256 slices, 8 to 32 columns
    // per workgroup and 128 to 512 workgroups all measured 3.96 - 4.2 us on the 7B layer (4 MB of partials).
    if (es == 4) launch_finalize_shape<4, 8, 32, 8>(partial, P, B, d, y, epoch, stream, ev_start, ev_stop, bias, fault);
    else launch_finalize_shape<2, 8, 32, 8>(partial, P, B, d, y, epoch, stream, ev_start, ev_stop, bias, fault);
}

// Ascending union index list, counts and per-token bit masks from the keep
// flags [B][F].  One workgroup of 1024 threads; all integer work.
__global__ void __launch_bounds__(1024)
k_ffn_lists(const unsigned char *__restrict__ keep, int B, int F, int32_t *__restrict__ active_idx,
            int32_t *__restrict__ n_active, uint32_t *__restrict__ mask_bits)
{
    // Pass 1, over (token, 32-flag word) pairs dealt to the threads round-robin (consecutive lanes =
    // consecutive words of one token, so the tokens' rows are read side by side instead of one after
    // the other): pack the flags into a mask word, OR it into the union word in LDS, count.
    // Pass 2: thread t owns the union words [t*wpt, (t+1)*wpt) and, after one workgroup-wide exclusive
    // scan of their popcounts, writes its neurons' indices in ascending order.
    __shared__ int s_wave[16];
    __shared__ int s_tok_cnt[CLADA_MAX_BATCH];
    __shared__ unsigned int s_uni[CLADA_MAX_DFF / 32];
    constexpr int MAXW = 8;                                   // words per thread: covers d_ff <= 262144
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int words = (F + 31) / 32;
    if (tid < CLADA_MAX_BATCH) s_tok_cnt[tid] = 0;
    for (int w = tid; w < words; w += 1024) s_uni[w] = 0u;
    __syncthreads();
    const int pairs = B * words;
    for (int idx0 = 0; idx0 < pairs; idx0 += 1024) {          // every lane stays in the loop: wave-wide sums below
        const int idx = idx0 + tid;
        const bool valid = idx < pairs;
        const int b = valid ? idx / words : B - 1, w = valid ? idx - b * words : 0;
        const unsigned char *row = keep + (size_t)b * F;
        unsigned int bits = 0u;
        const int j0 = 32 * w, nj = valid ? min(32, F - j0) : 0;
        if (nj == 32 && (reinterpret_cast<size_t>(row + j0) & 3) == 0) {
            // four flags per 32-bit load: high bit of every non-zero byte, gathered into a nibble
            // by a multiplication whose sixteen partial products all land on different bits
            const uint4 *r16 = reinterpret_cast<const uint4 *>(row + j0);
            unsigned int v[8];
            if ((reinterpret_cast<size_t>(r16) & 15) == 0) {
                const uint4 lo = r16[0], hi = r16[1];
                v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
            } else {
                const unsigned int *r4 = reinterpret_cast<const unsigned int *>(row + j0);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = r4[e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned int nz = ((((v[e] & 0x7f7f7f7fu) + 0x7f7f7f7fu) | v[e]) & 0x80808080u) >> 7;
                bits |= ((nz * 0x01020408u) >> 24) << (4 * e);
            }
        } else {
            for (int e = 0; e < nj; ++e) bits |= (row[j0 + e] != 0 ? 1u : 0u) << e;
        }
        if (mask_bits && valid) mask_bits[(size_t)b * words + w] = bits;
        if (bits) atomicOr(&s_uni[w], bits);
        // per-token counts: one LDS atomic per wave where the whole wave works on one token
        const int pc = __popc(bits);
        const int b0 = __builtin_amdgcn_readfirstlane(b);
        if (__all(b == b0)) {
            int t = pc;
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) t += __shfl_xor(t, o);
            if (lane == 0 && t) atomicAdd(&s_tok_cnt[b0], t);
        } else if (pc) {
            atomicAdd(&s_tok_cnt[b], pc);
        }
    }
    __syncthreads();
    const int wpt = (words + 1023) / 1024;
    const int w0 = min(words, tid * wpt), w1 = min(words, w0 + wpt);
    unsigned int uni[MAXW];
#pragma unroll
    for (int i = 0; i < MAXW; ++i) uni[i] = w0 + i < w1 ? s_uni[w0 + i] : 0u;
    int c = 0;
#pragma unroll
    for (int i = 0; i < MAXW; ++i) c += __popc(uni[i]);
    int inc = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    int base = 0, total = 0;
    for (int w = 0; w < 16; ++w) {
        const int v = s_wave[w];
        if (w < wave) base += v;
        total += v;
    }
    if (active_idx) {
        int pos = base + inc - c;
#pragma unroll
        for (int i = 0; i < MAXW; ++i) {
            unsigned int v = uni[i];
            while (v) {
                active_idx[pos++] = 32 * (w0 + i) + (__ffs(v) - 1);
                v &= v - 1u;
            }
        }
    }
    if (n_active) {
        if (tid == 0) n_active[0] = total;
        if (tid < B) n_active[1 + tid] = s_tok_cnt[tid];
    }
}


__device__ __forceinline__ int select_bit(unsigned long long m, int t)
{   // index of the t-th set bit of m (t < popcount(m))
    int i = 0;
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        const int c = __popcll(m & ((1ull << s) - 1ull));
        if (t >= c) { t -= c; m >>= s; i += s; }
    }
    return i;
}

// ---------------------------------------------------------------------------------------
// Split-d kernel for decode batch 1 (whole-KiB rows, <= 64 neurons per workgroup).
//   gate  : as above, one whole row per wave, next row prefetched while the current one is
//           reduced (loads never depend on a branch: out-of-range prefetches read x).
//   list  : every wave ballots the flags into the same ascending list (one barrier).
//   down  : the workgroup's kept neurons are taken DCH at a time.  Every wave owns a fixed
//           slice of the d columns (chunk c = wave, wave+NW, ...) and issues its 16-byte
//           loads of W_down[j, slice] for the whole chunk of neurons at once -- these loads
//           need only the list, not h, so up to DCH KiB per wave stream while ...
//   up    : ... the same waves take the chunk's W_up rows round-robin (two in flight),
//           h = a * (W_up[j,:].x) goes to LDS; after one barrier each wave adds
//           h * W_down[j, slice] into its 8 (bf16) or 4 (fp32) accumulators per chunk.
//   No cross-wave fold (each wave owns its columns) and plenty of bytes in flight, so a
//   workgroup with more kept neurons than its neighbours simply streams longer at its own rate.

struct B1Params {
    const char *wg, *wu, *wd, *x;
    const float *tau;
    float *partial;             // [P][d]
    unsigned char *keep;        // [F] or nullptr
    unsigned long long *rec;    // [P] keep mask (bit i = neuron blk + P*i, i < 56) | epoch tag in bits 56..63
    unsigned long long *apub;   // [P][64] published activations: fp32 bits | 32-bit call counter in the high half
    const unsigned int *epoch;  // device-side counter of balanced calls, advanced by k_ffn_finalize
                                // (read at kernel start, so graph replays stay correct)
    const float *b_in;          // RELU: input bias [F] or nullptr
    int *fault;                 // set to 1 when a balanced call gives up waiting for the other workgroups
    int max_spins;              // polls of the other workgroups' records before giving up
    int d, F, K0;
    int gelu;                   // gated family: sigma = tanh-form GELU instead of SiLU
    // Chained calls (whole-stack entry points): this launch also sums the partial outputs that the previous
    // launch of the chain left behind -- complete and visible, there is a kernel boundary in between -- so
    // that only the last layer of a chain needs a reduction launch of its own.
    const float *prev_partial;  // [P][d] of the previous launch, or nullptr
    char *prev_y;               // [d] output row of the previous layer
    const float *prev_bias;     // RELU: its output bias, or nullptr
    unsigned int *epoch_out;    // balanced calls of a chain advance the call counter themselves (no k_ffn_finalize does)
};

// Exclusive prefix sum over the 64 lanes of a wave (no barrier); *total gets the wave sum.
__device__ __forceinline__ int wave_excl_scan(int v, int lane, int *total)
{
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    *total = __shfl(inc, 63);
    return inc - v;
}

// ---- whole-stack variant: one persistent launch runs the L layers of a decode step (the future-work item
// "whole-stack persistence" next to mask compression).  Layers are independent problems (layer l has its own
// input row), so a workgroup that has finished its share of layer l goes straight on to the gate rows of
// layer l+1, and the fixed-order sum of the P partial outputs of layer l is done by all workgroups (each
// its own columns) in the middle of layer l+1, when every partial has long arrived: no kernel boundary and
// no separate reduction launch per layer.
#define CLADA_STACK_MAX_LAYERS 48
struct StackParams {
    const char *wg[CLADA_STACK_MAX_LAYERS], *wu[CLADA_STACK_MAX_LAYERS], *wd[CLADA_STACK_MAX_LAYERS];
    const float *b_in[CLADA_STACK_MAX_LAYERS], *b_out[CLADA_STACK_MAX_LAYERS];     // RELU only
    const char *x;              // [L][d]
    char *y;                    // [L][d]
    const float *tau;           // [L] (unused when DENSE)
    float *partial;             // [3][P][d], slot = layer number % 3
    unsigned long long *rec;    // [3][P] mask records / arrival records, slot = layer number % 3
    unsigned long long *apub;   // [2][P][64]
    unsigned int *epoch;        // layer numbers used up by the stack kernels of this context (advanced at kernel end)
    int *kcnt;                  // [3][P] kept neurons per workgroup
    int *n_active;              // [L][2] or nullptr
    int *fault;
    int max_spins, d, F, K0, gelu, L;
};

// The kernel reads these parameters through the kernel-argument segment's own address (constant address
// space, scalar loads): indexing the per-layer tables of a by-value copy with the running layer number made
// the compiler keep the whole copy in vector registers (+110 registers in every phase, spills in the hot loop).
typedef const __attribute__((address_space(4))) StackParams *StackArgs;

// Partial outputs cross workgroups inside one kernel: written through to memory (agent scope, the sc1 bit),
// read past the caches.  The language offers relaxed atomics of at most 64 bits for that, and four 8-byte
// write-through stores per 32 bytes turned every line of the partial into four partial-line writes; a whole
// 16-byte group goes out as one buffer store with the sc1 cache policy (16 in the builtin's last argument).
// (Written as inline assembly the same store lost data: the compiler cannot see that an asm statement is a
// store, so it did not keep the next write to the data registers away from it.)
__device__ __forceinline__ void store_through16(__amdgpu_buffer_rsrc_t row, int byte_off, float a, float b, float c, float d)
{
    const u32x4 v = {__float_as_uint(a), __float_as_uint(b), __float_as_uint(c), __float_as_uint(d)};
    __builtin_amdgcn_raw_buffer_store_b128(v, row, byte_off, 0, 16);
}
__device__ __forceinline__ float4 load_through(const float *src)
{
    const unsigned long long lo = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(src), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long hi = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(src) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float4(__uint_as_float((unsigned int)lo), __uint_as_float((unsigned int)(lo >> 32)),
                       __uint_as_float((unsigned int)hi), __uint_as_float((unsigned int)(hi >> 32)));
}

// y of stack layer l from the P partials, this workgroup's columns only, in the summation order of
// k_ffn_finalize (32 slices of P/32 partials each, then a fixed tree), so the result has the same bits as the
// per-layer call's.  A workgroup announces "my partial of layer l is in memory" with its record of layer l+1
// (published at the end of that layer's gate phase, when nothing of the workgroup is in flight any more), so
// once a workgroup holds all P records of layer l+1 it may read every partial of layer l.  The balanced
// kernel holds them anyway after its mask exchange; otherwise wave 0 reads them during the gate phase of
// layer l+2.  The reduction itself rides along with that gate phase in steps placed between the row loads,
// so that no trip through memory stops the stream of weight rows: (1) [wave 0, if not known yet] ask for the
// records, check them, tell the other waves through LDS, (2) ask for this thread's eight partial values,
// (3) add them, slice sum to LDS, and after the gate phase's barrier (4) the tree, the rounding and the
// store.  Partial buffers, kept counts and records rotate over three slots (layer number % 3): the record of
// the empty layer that ends a launch must not land on records a slower workgroup is still reading.
struct StackReduce {
    StackArgs pp;                   // the launch's parameters, read where needed (scalar loads)
    float4 (*s_sum)[16];
    volatile int *s_arrived;        // LDS: layer index (of this launch) whose preceding records are all in
    int P, d, G, cg, sl, col, slot, layer, wave;
    bool active;
    const unsigned long long *rec;  // records that confirm the partials wanted
    unsigned long long tag;
    unsigned long long m[4];
    bool asked;
    float4 v[8];
    int state;          // 0 waiting for the records, 2 partials asked, 3 slice sum in LDS (or nothing to do)

    __device__ __forceinline__ StackReduce(StackArgs pp_, float4 (*s)[16], volatile int *arr)
        : pp(pp_), s_sum(s), s_arrived(arr), asked(false), state(3) {}

    // reduction of the layer with number g, to be done inside launch-local layer `layer_now` (number g + 2)
    __device__ __forceinline__ void begin(unsigned int g, int layer_now, int tid, int wave_)
    {
        P = gridDim.x; d = pp->d;
        const int n4 = d / 4;
        G = (n4 + P - 1) / P;                               // float4 columns per workgroup (<= 16)
        cg = tid % G; sl = tid / G;
        col = ((int)blockIdx.x * G + cg) * 4;
        active = sl < 32 && col < d;
        slot = (int)(g % 3u);
        layer = layer_now; wave = wave_;
        rec = pp->rec + ((g + 1u) % 3u) * P;
        tag = (unsigned long long)((g + 2u) & 0xffu) << 56;     // tag of layer g + 1 = (its number + 1) & 255
        asked = false;
        // waves without a column of the reduction have nothing to load; wave 0 may still have to read records
        state = (wave * 64 < 32 * G || wave == 0) ? 0 : 3;
    }
    __device__ __forceinline__ void ask_records(int lane)
    {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = 4 * lane + u;
            m[u] = q < P ? __hip_atomic_load(rec + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : tag;
        }
        asked = true;
    }
    __device__ __forceinline__ bool records_ok() const
    {
        bool ok = true;
#pragma unroll
        for (int u = 0; u < 4; ++u) ok = ok && ((m[u] & (0xffull << 56)) == tag);
        return __ballot(ok) == ~0ull;
    }
    __device__ __forceinline__ void ask_partials()
    {
        const float *base = pp->partial + (size_t)slot * P * d + col;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int q = sl + 32 * u;
            v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (active && q < P) v[u] = load_through(base + (size_t)q * d);
        }
        state = 2;
    }
    __device__ __forceinline__ void add_partials()
    {
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 8; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
        if (sl < 32) s_sum[sl][cg] = s;
        state = 3;
    }
    // one step per call, never waits (the caller places the calls between its own loads)
    __device__ __forceinline__ void step(int lane)
    {
        if (state == 0) {
            if (*s_arrived == layer) {
                ask_partials();
            } else if (wave == 0) {
                if (asked && records_ok()) {
                    if (lane == 0) *s_arrived = layer;
                    ask_partials();
                } else {
                    ask_records(lane);
                }
            }
        } else if (state == 2) {
            add_partials();
        }
    }
    // whatever is left, waiting (bounded) where it must
    __device__ __forceinline__ void finish(int lane)
    {
        if (state == 0) {
            if (*s_arrived != layer) {
                if (wave == 0) {
                    bool ok = asked && records_ok();
                    for (int spins = 0; spins <= pp->max_spins && !ok; ++spins) {
                        ask_records(lane);
                        ok = records_ok();
                        if (!ok) __builtin_amdgcn_s_sleep(8);
                    }
                    if (lane == 0) {
                        if (!ok) __hip_atomic_store(pp->fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        *s_arrived = layer;
                    }
                } else {
                    // wave 0 sets the flag in every case, at the latest at the end of its own gate rows
                    for (int spins = 0; spins < (1 << 24) && *s_arrived != layer; ++spins) __builtin_amdgcn_s_sleep(2);
                    if (*s_arrived != layer && lane == 0) __hip_atomic_store(pp->fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            ask_partials();
        }
        if (state == 2) add_partials();
    }
    // after a workgroup barrier that follows finish(): tree over the 32 slices, rounding, store of y[l]
    template <int ES, bool RELU>
    __device__ __forceinline__ void tree_and_store(int l, int tid)
    {
        const int lane = tid & 63;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        if (sl < 32) s = s_sum[sl][cg];
#pragma unroll
        for (int h = 16; h >= 1; h >>= 1) {
            if (sl < h) {
                const float4 w = s_sum[sl + h][cg];
                s.x += w.x; s.y += w.y; s.z += w.z; s.w += w.w;
                s_sum[sl][cg] = s;
            }
            __syncthreads();
        }
        if (sl == 0 && col < d) {
            if (__hip_atomic_load(pp->fault, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) s.x = s.y = s.z = s.w = __int_as_float(0x7fc00000);
            if (RELU && pp->b_out[l]) {
                const float4 bv = *reinterpret_cast<const float4 *>(pp->b_out[l] + col);
                s.x += bv.x; s.y += bv.y; s.z += bv.z; s.w += bv.w;
            }
            char *y = pp->y + (size_t)l * d * ES;
            if (ES == 4) {
                *reinterpret_cast<float4 *>(y + (size_t)col * 4) = s;
            } else {
                uint2 o;
                o.x = f32_to_bf16_bits(s.x) | (f32_to_bf16_bits(s.y) << 16);
                o.y = f32_to_bf16_bits(s.z) | (f32_to_bf16_bits(s.w) << 16);
                *reinterpret_cast<uint2 *>(y + (size_t)col * 2) = o;
            }
        }
        // kept neurons of the layer: the workgroups' counts, summed by one wave of workgroup 0
        if (pp->n_active && blockIdx.x == 0 && tid >= 64 && tid < 128) {
            int c = 0;
            for (int q = lane; q < P; q += 64) c += __hip_atomic_load(pp->kcnt + slot * P + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) c += __shfl_xor(c, o);
            if (lane == 0) { pp->n_active[2 * l] = c; pp->n_active[2 * l + 1] = c; }
        }
        state = 3;
    }
};

struct NoStackReduce {       // the per-layer kernel has nothing to ride along
    template <typename P, typename S, typename A> __device__ __forceinline__ NoStackReduce(const P &, S, A) {}
};

// BAL = cross-workgroup load balancing (sparse calls): a workgroup's kept count is binomial, and
// measured per-workgroup timelines show the busiest workgroup finishing ~5 us after the average
// one.  After the gate phase every workgroup publishes its keep mask (<= 56 neurons -> one 64-bit
// word with an 8-bit epoch tag) and its activations with agent-scope write-through stores, takes
// its own first K0 kept neurons as chunk 0, and while those loads stream wave 0 alone reads all P
// masks, prefix-sums them and hands the workgroup its share of the pooled surplus, so that every
// workgroup ends up with floor/ceil(k/P) neurons.  The assignment is a function of the masks
// only: summation order and result stay bit-reproducible.  Needs all P workgroups co-resident.
// (A variant that also ran the cross-workgroup reduction of the partial y's inside this kernel --
// write-through partials, "done" tags, every workgroup adding its d/P columns -- was measured
// 7 us slower than the separate k_ffn_finalize launch: each agent-scope round trip costs ~3 us
// here.  For the same reason balancing only pays when chunk 0 is long enough to hide two hops.)
// RELU: the non-gated family -- no W_up rows at all, h is the activation itself.
// STACK: the whole-stack variant described above (parameters StackParams; the per-layer state below is
// rebuilt from them at the top of every layer).
// ROUNDS: more than 64 neurons per workgroup, worked off 64 at a time (a template flag: an enclosing loop
// of unknown trip count costs the kernel ~50 registers, which the balanced instances do not have).
// OCC2: an instance for the lanes of the whole-stack calls that fits two workgroups on a compute unit (at most 128
// registers per lane: x in LDS, DCH = 8), so that a workgroup of layer l and one of layer l+1 share every unit and
// one's gate phase runs under the other's kept-row phase.
template <int ES, int NCH, int NW, int DCH, bool DENSE, bool BAL, bool RELU = false, bool STACK = false, bool ROUNDS = false,
          bool OCC2 = false>
__global__ void __launch_bounds__(NW * 64, OCC2 ? 4 : 1)
k_ffn_decode_b1(const std::conditional_t<STACK, StackParams, B1Params> pp)
{
    constexpr int VEC = 16 / ES;
    constexpr int ROWB = NCH * 1024;
    constexpr int SL = (NCH + NW - 1) / NW;                 // column chunks owned by a wave
    constexpr int UPB = (DCH + NW - 1) / NW;                // W_up rows a wave takes per chunk
    // own-first chunk: two W_up rows for waves 1..NW-1 (one with 10 KiB rows, which would not fit the registers)
    constexpr int K0MAX = (NCH > 8 ? 1 : 2) * (NW - 1);
    // x in LDS instead of registers: the whole-stack kernel, and rows of 12 and 16 KiB (two row buffers of the
    // gate phase alone are 96 / 128 registers there)
    constexpr bool XLDS = STACK || NCH > 10 || OCC2;
    static_assert(!(DENSE && BAL), "the dense twin needs no balancing");
    static_assert(!(ROUNDS && (BAL || STACK)), "rounds only in the plain split-d kernel");
    static_assert(!(OCC2 && (BAL || STACK || ROUNDS)), "the two-per-unit instance is a plain split-d kernel");
    __shared__ float s_a[64];
    __shared__ int s_flag[64];
    __shared__ int s_list[64];
    __shared__ float s_h[2][DCH > K0MAX ? DCH : K0MAX];
    __shared__ int s_l2row[64];                             // balanced share: weight row ...
    __shared__ int s_l2a[64];                               // ... and index of its published activation
    __shared__ int s_n2;
    __shared__ float4 s_sum[STACK ? 32 : 1][16];            // STACK: slices of the final reduction
    __shared__ int s_arrived;                               // STACK: see StackReduce
    __shared__ __align__(16) unsigned char s_x[(STACK || NCH > 10 || OCC2) ? NCH * 1024 : 16];    // the layer's input row where it is not held in registers
    // chained calls: this workgroup's CGW column groups (of four) of all 256 partial outputs of the previous launch
    constexpr int CGW = (NCH * 1024 / ES / 4 + 255) / 256;
    __shared__ float4 s_prev[STACK ? 1 : 256 * CGW];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int blk = blockIdx.x, P = gridDim.x;
    StackArgs ka = nullptr;
    int F;
    if constexpr (STACK) {
        ka = (StackArgs)__builtin_amdgcn_kernarg_segment_ptr();    // = pp, the only argument
        F = ka->F;
    } else {
        F = pp.F;
    }
    const int ni_all = blk < F ? (F - blk + P - 1) / P : 0; // this workgroup's neurons: blk, blk + P, ... (<= 56 when BAL)

    const int loff = lane * 16;
    unsigned int g0 = 0u;                                   // STACK: number of this launch's first layer on the context
    int n_layers = 1;
    if constexpr (STACK) {
        g0 = *ka->epoch;
        n_layers = ka->L;
        if (threadIdx.x == 0) s_arrived = -1;               // first read two layers (many barriers) from here
    }
#pragma clang loop unroll(disable)
  for (int layer = 0; layer < n_layers; ++layer) {
    // STACK: the lane-dependent values are made opaque per layer, or the compiler hoists every address
    // offset derived from them out of the loop and holds ~50 more registers across the whole body
    int tid_l = threadIdx.x;
    if constexpr (STACK) asm volatile("" : "+v"(tid_l));
    const int tid = tid_l, lane = tid & 63, loff = lane * 16;
    B1Params p;
    if constexpr (STACK) {
        const unsigned int g = g0 + (unsigned int)layer;
        p.wg = ka->wg[layer]; p.wu = ka->wu[layer]; p.wd = ka->wd[layer];
        p.x = ka->x + (size_t)layer * ROWB;
        p.tau = ka->tau + layer;
        p.partial = ka->partial + (size_t)(g % 3u) * P * ka->d;
        p.keep = nullptr;
        p.rec = ka->rec + (g % 3u) * P;
        p.apub = ka->apub + (size_t)(g & 1u) * P * 64;
        p.epoch = nullptr;
        p.b_in = RELU ? ka->b_in[layer] : nullptr;
        p.fault = ka->fault;
        p.max_spins = ka->max_spins;
        p.d = ka->d; p.F = F; p.K0 = ka->K0; p.gelu = ka->gelu;
        p.prev_partial = nullptr; p.prev_y = nullptr; p.prev_bias = nullptr; p.epoch_out = nullptr;
    } else {
        p = pp;
    }
    (void)ka;

    auto load_row = [&](u32x4 (&buf)[NCH], const char *w, int j) {
        const char *row = w + (size_t)j * ROWB + loff;
#pragma unroll
        for (int c = 0; c < NCH; ++c) buf[c] = ld_stream16(row + c * 1024);
    };

    float acc[SL][VEC];
#pragma unroll
    for (int s = 0; s < SL; ++s)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[s][e] = 0.0f;

    // More than 64 neurons per workgroup (d_ff above 64 P: the 70B-class layers) are worked off in rounds of
    // 64, gate rows and kept rows of a round before the next round's; the accumulators run through.  (The
    // balanced and the whole-stack variants are only launched where one round covers everything.)
    unsigned long long tag = 0ull;
    unsigned int call_no = 0u;                              // this balanced call's number on the context
    if (BAL || STACK) {
        if constexpr (STACK) call_no = g0 + (unsigned int)layer + 1u;
        else call_no = *p.epoch + 1u;
        tag = (unsigned long long)(call_no & 0xffu) << 56;
    }
    // (read here, not where it is used: at the kernel's end the round trip would be exposed)
    int prev_fault = 0;
    if constexpr (!STACK && BAL) {
        if (p.prev_partial) prev_fault = *p.fault;
    }
    // Chained call: the previous launch's partial outputs for this workgroup's columns go straight into LDS
    // (no staging registers; a wave's transfer fills 64 consecutive 16-byte entries, entry e = partial
    // e / CGW, column group e % CGW) and are summed at the very end of this kernel.  (Measured on the 7B
    // layer: the transfers cost the kernel 1.1 us, the sum 0.3 us, against 2.9 us for a reduction launch.)
    auto prefetch_prev = [&]() {
        const int d4 = p.d >> 2;
        for (int e0 = wave * 64; e0 < 256 * CGW; e0 += NW * 64) {
            const int e = e0 + lane;
            const int q = e / CGW, cg4 = min(blk * CGW + e % CGW, d4 - 1);
            __builtin_amdgcn_global_load_lds(
                (const void __attribute__((address_space(1))) *)(p.prev_partial + (size_t)q * p.d + 4 * cg4),
                (void __attribute__((address_space(3))) *)(s_prev + e0), 16, 0, 0);
        }
    };
    if constexpr (!STACK) {
        if (p.prev_partial) prefetch_prev();
    }
   for (int r0 = 0; r0 < (ROUNDS ? ni_all : 1); r0 += 64) {
    const int ni = ROUNDS ? min(64, ni_all - r0) : ni_all;
    const int nb0 = blk + P * r0;                           // the round's first neuron
    // first gate row on its way before anything else
    u32x4 ga[NCH], gb[NCH];
    if (wave < ni) load_row(ga, p.wg, nb0 + P * wave);
    // x: held packed in registers; where there is less room (XLDS) it sits in LDS and a chunk is read where it is used
    u32x4 xr[XLDS ? 1 : NCH];
    if constexpr (XLDS) {
        for (int o = tid * 16; o < ROWB; o += NW * 64 * 16)
            *reinterpret_cast<u32x4 *>(s_x + o) = *reinterpret_cast<const u32x4 *>(p.x + o);
        __syncthreads();
    } else {
#pragma unroll
        for (int c = 0; c < NCH; ++c) xr[c] = *reinterpret_cast<const u32x4 *>(p.x + c * 1024 + loff);
    }
    auto xv = [&](int c) -> u32x4 {
        if constexpr (XLDS) return *reinterpret_cast<const u32x4 *>(s_x + c * 1024 + loff);
        else return xr[c];
    };
    const float tau = DENSE ? 0.0f : p.tau[0];
    // An activation another workgroup published: the word carries the number of the call that wrote it, so
    // it validates itself and needs no ordering against the mask record that announced it.  Bounded like the
    // wait for the records (the store was issued before the record's, so a second poll is already rare).
    auto published_act = [&](int slot) -> float {
        unsigned long long v = 0ull;
        bool ok = false;
        for (int spins = 0; spins <= p.max_spins && !ok; ++spins) {
            v = __hip_atomic_load(p.apub + slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ok = (unsigned int)(v >> 32) == call_no;
        }
        if (!ok) {
            __hip_atomic_store(p.fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return 0.0f;
        }
        return __uint_as_float((unsigned int)v);
    };

    auto gate_finish = [&](const u32x4 (&buf)[NCH], int i) {
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) s = dot16<ES>(buf[c], xv(c), s);
        s = wave_sum(s);
        const float a = ffn_act<RELU>(s, p.b_in, (size_t)(nb0 + P * i), p.gelu);
        const bool keep = DENSE ? true : (fabsf(a) >= tau);
        if (lane == 0) {
            s_a[i] = a;
            s_flag[i] = keep ? 1 : 0;
            if (p.keep) p.keep[nb0 + P * i] = keep ? 1 : 0;
        }
    };
    // STACK: the final reduction of the layer before the previous one rides along with this gate phase
    std::conditional_t<STACK, StackReduce, NoStackReduce> red(ka, s_sum, &s_arrived);
    if constexpr (STACK) {
        if (layer >= 2) red.begin(g0 + (unsigned int)layer - 2u, layer, tid, wave);
    }
    // ---------------------------------------------------------------- gate phase: the next row is
    // requested before the current one is reduced; every path has a fixed number of loads in flight
    for (int i = wave; i < ni; i += 2 * NW) {
        if constexpr (STACK) red.step(lane);
        if (i + NW < ni) {
            load_row(gb, p.wg, nb0 + P * (i + NW));
            gate_finish(ga, i);
            if (i + 2 * NW < ni) {
                load_row(ga, p.wg, nb0 + P * (i + 2 * NW));
                gate_finish(gb, i + NW);
            } else {
                gate_finish(gb, i + NW);
            }
        } else {
            gate_finish(ga, i);
        }
    }
    if constexpr (STACK) {
        if (layer >= 2) red.finish(lane);
        // nothing of this wave is in flight any more, so the write-through stores of the previous layer's
        // partial have been acknowledged by memory (the vector-memory counter at zero says exactly that for
        // stores that bypass the caches): after the barrier that partial is announced.  A release fence at
        // agent scope would do the same formally, but it writes the whole L2 back (+9.5 us per layer measured).
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();
    if constexpr (STACK) {
        // the record of this layer doubles as "my partial of the previous layer is in memory"; the balanced
        // kernel publishes it with its mask below
        if (!BAL && tid == 0) __hip_atomic_store(p.rec + blk, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (layer >= 2) red.template tree_and_store<ES, RELU>(layer - 2, tid);
    }

    // every wave derives the same ascending list
    const unsigned long long mask = __ballot(lane < ni && s_flag[lane] != 0);
    const int kp = __popcll(mask);
    if constexpr (STACK && !DENSE) {
        if (ka->n_active && tid == 0)
            __hip_atomic_store(ka->kcnt + ((g0 + (unsigned int)layer) % 3u) * P + blk, kp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if ((mask >> lane) & 1ull) s_list[__popcll(mask & ((1ull << lane) - 1ull))] = lane;

    // h * W_down[j, slice] for one chunk of neurons, straight from the loaded registers
    auto down_fma = [&](auto dnc, const u32x4 (&dn)[decltype(dnc)::value][SL], const float *hs, int nvalid) {
        constexpr int N = decltype(dnc)::value;
#pragma unroll
        for (int e = 0; e < N; ++e) {
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
    auto down_load = [&](auto dnc, u32x4 (&dn)[decltype(dnc)::value][SL], const int *rows, int nvalid, bool local) {
        constexpr int N = decltype(dnc)::value;
#pragma unroll
        for (int e = 0; e < N; ++e) {
            if (e < nvalid) {
                const int j = local ? nb0 + P * rows[e] : rows[e];
#pragma unroll
                for (int s = 0; s < SL; ++s) {
                    const int c = wave + s * NW;
                    if (c < NCH) dn[e][s] = ld_stream16(p.wd + (size_t)j * ROWB + c * 1024 + loff);
                    else dn[e][s] = u32x4{0u, 0u, 0u, 0u};
                }
            } else {
#pragma unroll
                for (int s = 0; s < SL; ++s) dn[e][s] = u32x4{0u, 0u, 0u, 0u};
            }
        }
    };
    // R W_up rows of this wave in flight together: entries first, first+stride, ... of a list
    auto up_rows = [&](auto rc, const int *rows, const int *aidx, bool local, int first, int stride, float *hs) {
        constexpr int R = decltype(rc)::value;
        u32x4 up[R][NCH];
        float av[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int e = first + r * stride;
            const int j = local ? nb0 + P * rows[e] : rows[e];
            if (local) av[r] = s_a[rows[e]];
            else av[r] = published_act(aidx[e]);
            if (!RELU) load_row(up[r], p.wu, j);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float s0 = 1.0f;
            if (!RELU) {
                s0 = 0.0f;
#pragma unroll
                for (int c = 0; c < NCH; ++c) s0 = dot16<ES>(up[r][c], xv(c), s0);
                s0 = wave_sum(s0);
            }
            if (lane == 0) hs[first + r * stride] = RELU ? av[r] : av[r] * s0;
        }
    };

    int par = 0;
    if (BAL) {
        // ------------------------------------------------ publish, then chunk 0 = own first K0 neurons
        const int K0 = min(p.K0, K0MAX);
        const int own = min(kp, K0);
        if (wave == 0) {
            // Every published word is one 64-bit atomic object that names the call it belongs to (the mask
            // record by an 8-bit tag -- every call rewrites every record --, an activation by the full call
            // number), so readers never pair a fresh word with a stale one and no release/acquire is needed.
            // (An agent-scope release here writes back the XCD's L2: measured +9.5 us per call.)
            if (lane < ni)
                __hip_atomic_store(p.apub + blk * 64 + lane,
                                   ((unsigned long long)call_no << 32) | __float_as_uint(s_a[lane]),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (lane == 0) __hip_atomic_store(p.rec + blk, mask | tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        u32x4 dn0[K0MAX][SL];
        down_load(std::integral_constant<int, K0MAX>{}, dn0, s_list, own, true);
        if (wave > 0) {                                     // W_up rows of chunk 0 go to waves 1..NW-1
            const int first = wave - 1;
            const int nup = first < own ? (own - first + NW - 2) / (NW - 1) : 0;
            if (nup == 1) up_rows(std::integral_constant<int, 1>{}, s_list, nullptr, true, first, NW - 1, s_h[0]);
            else if (nup == 2) up_rows(std::integral_constant<int, K0MAX >= 2 * (NW - 1) ? 2 : 1>{}, s_list, nullptr, true, first, NW - 1, s_h[0]);
        } else {
            // wave 0: read all P masks (lane handles records 4*lane .. 4*lane+3), no barriers
            // The wait is bounded: if the other workgroups' records do not arrive (they can only be
            // missing while something else holds the compute units they need, e.g. a second balanced
            // call overlapping from another stream), this workgroup gives up its share, raises the
            // context's fault flag, and the final reduction turns the output into NaN.
            unsigned long long m[4];
            bool gave_up = false;
            for (int spins = 0;; ++spins) {
                if (spins >= p.max_spins) { gave_up = true; break; }
                bool ok = true;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = 4 * lane + u;
                    m[u] = q < P ? __hip_atomic_load(p.rec + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : tag;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) ok = ok && ((m[u] & (0xffull << 56)) == tag);
                if (__ballot(ok) == ~0ull) break;
                __builtin_amdgcn_s_sleep(8);
            }
            if (gave_up) {
                if (lane == 0) {
                    s_n2 = 0;
                    __hip_atomic_store(p.fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            } else {
            int kq[4], oq[4], sq[4], ksum = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                m[u] &= ~(0xffull << 56);
                kq[u] = __popcll(m[u]);
                oq[u] = min(kq[u], K0);
                sq[u] = kq[u] - oq[u];
                ksum += kq[u];
            }
            int K;
            (void)wave_excl_scan(ksum, lane, &K);
            // target of workgroup q: floor((q+1)K/P) - floor(qK/P); extra = target - own-first, >= 0
            int eq[4], se = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = 4 * lane + u;
                const int tgt = q < P ? (int)(((long long)(q + 1) * K) / P - ((long long)q * K) / P) : 0;
                eq[u] = max(0, tgt - oq[u]);
                se += sq[u] | (eq[u] << 16);
            }
            int SE;
            int pre = wave_excl_scan(se, lane, &SE);        // surplus prefix (low half) | extra prefix (high half)
            const int S = SE & 0xffff;
            // this workgroup's slice [lo, hi) of the pooled surplus
            int spre[4], epre[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                spre[u] = pre & 0xffff;
                epre[u] = pre >> 16;
                pre += sq[u] | (eq[u] << 16);
            }
            int lo_l = 0, hi_l = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (4 * lane + u == blk) { lo_l = min(epre[u], S); hi_l = min(epre[u] + eq[u], S); }
            const int lo = __shfl(lo_l, blk >> 2), hi = __shfl(hi_l, blk >> 2);
            // record q hands over the part of its surplus [spre, spre+sq) that falls into [lo, hi)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = 4 * lane + u;
                const int a0 = max(lo, spre[u]), a1 = min(hi, spre[u] + sq[u]);
                for (int r = a0; r < a1; ++r) {
                    const int i = select_bit(m[u], oq[u] + (r - spre[u]));
                    s_l2row[r - lo] = q + P * i;
                    s_l2a[r - lo] = q * 64 + i;
                }
            }
            if (lane == 0) s_n2 = hi - lo;
            }
            if constexpr (STACK) {
                if (lane == 0) s_arrived = layer + 1;      // all records of this layer seen (or given up, flagged)
            }
        }
        __syncthreads();
        // first chunk of the balanced share: its loads go out before chunk 0 is consumed
        const int n2 = s_n2;
        {
            const int nc = min(DCH, n2);
            u32x4 dn[DCH][SL];
            down_load(std::integral_constant<int, DCH>{}, dn, s_l2row, nc, false);
            const int nup = wave < nc ? (nc - wave + NW - 1) / NW : 0;
            // W_up rows requested now, reduced after chunk 0's accumulation
            u32x4 up[UPB][NCH];
            float av[UPB];
#pragma unroll
            for (int r = 0; r < UPB; ++r)
                if (r < nup) {
                    const int e = wave + r * NW;
                    av[r] = published_act(s_l2a[e]);
                    if (!RELU) load_row(up[r], p.wu, s_l2row[e]);
                }
            down_fma(std::integral_constant<int, K0MAX>{}, dn0, s_h[0], own);
#pragma unroll
            for (int r = 0; r < UPB; ++r)
                if (r < nup) {
                    float s0 = 1.0f;
                    if (!RELU) {
                        s0 = 0.0f;
#pragma unroll
                        for (int c = 0; c < NCH; ++c) s0 = dot16<ES>(up[r][c], xv(c), s0);
                        s0 = wave_sum(s0);
                    }
                    if (lane == 0) s_h[1][wave + r * NW] = RELU ? av[r] : av[r] * s0;
                }
            __syncthreads();
            down_fma(std::integral_constant<int, DCH>{}, dn, s_h[1], nc);
        }
        // rest of the share (rare: more than DCH extra neurons)
        par = 0;
        for (int c0 = DCH; c0 < n2; c0 += DCH, par ^= 1) {
            const int nc = min(DCH, n2 - c0);
            u32x4 dn[DCH][SL];
            down_load(std::integral_constant<int, DCH>{}, dn, s_l2row + c0, nc, false);
            const int nup = wave < nc ? (nc - wave + NW - 1) / NW : 0;
            if (nup == 1) up_rows(std::integral_constant<int, 1>{}, s_l2row + c0, s_l2a + c0, false, wave, NW, s_h[par]);
            else if (nup == 2) up_rows(std::integral_constant<int, UPB >= 2 ? 2 : 1>{}, s_l2row + c0, s_l2a + c0, false, wave, NW, s_h[par]);
            else if (nup == 3) up_rows(std::integral_constant<int, UPB >= 3 ? 3 : 1>{}, s_l2row + c0, s_l2a + c0, false, wave, NW, s_h[par]);
            __syncthreads();
            down_fma(std::integral_constant<int, DCH>{}, dn, s_h[par], nc);
        }
    } else {
        // ------------------------------------------------ no balancing: the workgroup's own list, DCH at a time
        for (int c0 = 0; c0 < kp; c0 += DCH, par ^= 1) {
            const int nc = min(DCH, kp - c0);
            u32x4 dn[DCH][SL];
            down_load(std::integral_constant<int, DCH>{}, dn, s_list + c0, nc, true);
            const int nup = wave < nc ? (nc - wave + NW - 1) / NW : 0;
            static_assert(UPB <= 3, "add cases");
            if (nup == 1) up_rows(std::integral_constant<int, 1>{}, s_list + c0, nullptr, true, wave, NW, s_h[par]);
            else if (nup == 2) up_rows(std::integral_constant<int, UPB >= 2 ? 2 : 1>{}, s_list + c0, nullptr, true, wave, NW, s_h[par]);
            else if (nup == 3) up_rows(std::integral_constant<int, UPB >= 3 ? 3 : 1>{}, s_list + c0, nullptr, true, wave, NW, s_h[par]);
            __syncthreads();
            down_fma(std::integral_constant<int, DCH>{}, dn, s_h[par], nc);
        }
    }
    if (ROUNDS && r0 + 64 < ni_all) __syncthreads();       // the LDS arrays are free for the next round
   }    // rounds
    if constexpr (!STACK) {
        if (p.prev_partial) {
            // chained call: this wave's transfers of the previous partials have landed (its other loads are
            // long consumed, nothing else is in flight); after the barrier all of them have
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
    }
    // each wave owns its columns: straight to the partial, no fold
    float *dst = p.partial + (size_t)blk * p.d;
    __amdgpu_buffer_rsrc_t dst_row = __builtin_amdgcn_make_buffer_rsrc(dst, 0, p.d * 4, 0x00020000);   // raw bytes, bounds = the row
#pragma unroll
    for (int s = 0; s < SL; ++s) {
        const int c = wave + s * NW;
        if (c < NCH) {
#pragma unroll
            for (int k = 0; k < VEC; k += 4) {
                if constexpr (STACK) {
                    store_through16(dst_row, ((c * 64 + lane) * VEC + k) * 4, acc[s][k], acc[s][k + 1], acc[s][k + 2], acc[s][k + 3]);
                } else {
                    *reinterpret_cast<float4 *>(dst + (c * 64 + lane) * VEC + k) =
                        make_float4(acc[s][k], acc[s][k + 1], acc[s][k + 2], acc[s][k + 3]);
                }
            }
        }
    }
    if constexpr (STACK) __syncthreads();          // the LDS arrays are free for the next layer
    if constexpr (!STACK) {
        if (p.prev_partial) {
            // y of the previous layer = sum of its 256 partials in k_ffn_finalize's order (the bits match):
            // slice sl adds the partials sl, sl + 32, ... one after the other, then the 32 slices fold by the
            // fixed tree sl += sl + 16, 8, 4, 2, 1.  A column group's 32 slices sit in one half of a wave.
            if (tid < 32 * CGW) {
                const int sl = tid & 31, cg = tid >> 5;
                float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const float4 v = s_prev[(sl + 32 * u) * CGW + cg];
                    t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
                }
#pragma unroll
                for (int h = 16; h >= 1; h >>= 1) {
                    const float vx = __shfl_down(t.x, h, 32), vy = __shfl_down(t.y, h, 32);
                    const float vz = __shfl_down(t.z, h, 32), vw = __shfl_down(t.w, h, 32);
                    if (sl < h) { t.x += vx; t.y += vy; t.z += vz; t.w += vw; }
                }
                const int col = (blk * CGW + cg) * 4;
                if (sl == 0 && col < p.d) {
                    if (prev_fault) t.x = t.y = t.z = t.w = __int_as_float(0x7fc00000);   // a balanced call gave up: no silent wrong sums
                    if (RELU && p.prev_bias) {
                        const float4 bv = *reinterpret_cast<const float4 *>(p.prev_bias + col);
                        t.x += bv.x; t.y += bv.y; t.z += bv.z; t.w += bv.w;
                    }
                    if (ES == 4) {
                        *reinterpret_cast<float4 *>(p.prev_y + (size_t)col * 4) = t;
                    } else {
                        uint2 o;
                        o.x = f32_to_bf16_bits(t.x) | (f32_to_bf16_bits(t.y) << 16);
                        o.y = f32_to_bf16_bits(t.z) | (f32_to_bf16_bits(t.w) << 16);
                        *reinterpret_cast<uint2 *>(p.prev_y + (size_t)col * 2) = o;
                    }
                }
            }
        }
        // every workgroup of a balanced call has read the counter before workgroup 0 gets past the mask exchange
        if (BAL && p.epoch_out && blk == 0 && tid == 0) *p.epoch_out = call_no;
    }
  }     // layers
    if constexpr (STACK) {
        // drain: a record of one more (empty) layer announces the last partial, then the two reductions still owed
        const int tid = threadIdx.x, lane = tid & 63;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        const unsigned int g_end = g0 + (unsigned int)n_layers;
        if (tid == 0)
            __hip_atomic_store(ka->rec + (g_end % 3u) * P + blk, (unsigned long long)((g_end + 1u) & 0xffu) << 56,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        StackReduce red(ka, s_sum, &s_arrived);
        for (int l = n_layers >= 2 ? n_layers - 2 : 0; l < n_layers; ++l) {
            // both wait for the records of the empty layer: those confirm every earlier partial of their senders
            red.begin(g0 + (unsigned int)l, n_layers + 1, tid, wave);
            red.rec = ka->rec + (g_end % 3u) * P;
            red.tag = (unsigned long long)((g_end + 1u) & 0xffu) << 56;
            red.finish(lane);
            __syncthreads();
            red.template tree_and_store<ES, RELU>(l, tid);
        }
        // the empty layer uses up a number too (its records must not be mistaken for the next launch's first
        // layer); every workgroup has read the counter at its start: they all sent that record
        if (blk == 0 && tid == 0) *ka->epoch = g_end + 1u;
    }
}

template <int ES, int NCH, int DCH, bool DENSE, bool BAL, bool RELU = false>
hipError_t launch_b1_variant(clada_ctx *ctx, const B1Params &p, int P, hipStream_t st)
{
    const bool rounds = (p.F + P - 1) / P > 64;
    if constexpr (BAL) { if (rounds) return hipErrorNotSupported; }
    auto kern = (!BAL && rounds) ? k_ffn_decode_b1<ES, NCH, 8, DCH, DENSE, false, RELU, false, !BAL>
                                 : k_ffn_decode_b1<ES, NCH, 8, DCH, DENSE, BAL, RELU>;
    if (BAL) {          // spinning on other workgroups' records needs every workgroup resident at once
        // (the answer is kept in the context: it belongs to the context's device, and a context is used by
        // one thread at a time)
        const void *fn = reinterpret_cast<const void *>(kern);
        int occ = -1;
        for (int i = 0; i < ctx->n_occ; ++i)
            if (ctx->occ_fn[i] == fn) occ = ctx->occ_val[i];
        if (occ < 0) {
            int nb = 0;
            hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, 512, 0);
            if (e != hipSuccess) return e;
            occ = nb;
            if (ctx->n_occ < CLADA_OCC_SLOTS) {
                ctx->occ_fn[ctx->n_occ] = fn;
                ctx->occ_val[ctx->n_occ++] = nb;
            }
        }
        if ((long long)occ * ctx->num_cu < P) return hipErrorNotSupported;
    }
    // with the diagnostic option on, the two events take the kernel's own start and stop times
    if (ctx->opt_diag_events) hipExtLaunchKernelGGL(kern, dim3(P), dim3(512), 0, st, ctx->ev[0], ctx->ev[1], 0, p);
    else hipLaunchKernelGGL(kern, dim3(P), dim3(512), 0, st, p);
    return hipGetLastError();
}

template <int ES, int NCH, int DCH, bool RELU = false>
hipError_t launch_b1(clada_ctx *ctx, const B1Params &p, int P, bool dense, bool balance, hipStream_t st)
{
    if (dense) return launch_b1_variant<ES, NCH, DCH, true, false, RELU>(ctx, p, P, st);
    if (balance) return launch_b1_variant<ES, NCH, DCH, false, true, RELU>(ctx, p, P, st);
    return launch_b1_variant<ES, NCH, DCH, false, false, RELU>(ctx, p, P, st);
}

// The two-per-unit instances (bf16, one round of neurons), sparse or dense; false where the shape has none.
template <int NCH, int DCH, bool RELU>
hipError_t launch_b1_occ2_shape(const B1Params &p, int P, bool dense, hipStream_t st)
{
    if (dense) hipLaunchKernelGGL((k_ffn_decode_b1<2, NCH, 8, DCH, true, false, RELU, false, false, true>), dim3(P), dim3(512), 0, st, p);
    else hipLaunchKernelGGL((k_ffn_decode_b1<2, NCH, 8, DCH, false, false, RELU, false, false, true>), dim3(P), dim3(512), 0, st, p);
    return hipGetLastError();
}

bool b1_occ2_shape_ok(int es, int nch, bool relu)
{
    // (10 KiB rows: the instance needs 128 registers and a few spills, and was measured 6 % slower than the
    // one-per-unit instance in two lanes)
    return es == 2 && (relu ? nch == 5 : (nch == 4 || nch == 8));
}

hipError_t launch_b1_occ2(const B1Params &p, int P, int nch, bool relu, bool dense, hipStream_t st)
{
    if (relu) return launch_b1_occ2_shape<5, 8, true>(p, P, dense, st);
    if (nch == 4) return launch_b1_occ2_shape<4, 8, false>(p, P, dense, st);
    return launch_b1_occ2_shape<8, 8, false>(p, P, dense, st);
}

// The split-d instantiations by element size, row length and family (exactly the shapes b1_shape_ok admits).
// *balance is cleared when the balanced instance cannot have all its workgroups resident at once.
bool b1_shape_ok(int es, int nch, bool relu)
{
    return relu ? (es == 2 && (nch == 2 || nch == 5 || nch == 8 || nch == 10))
           : es == 2 ? (nch == 2 || nch == 4 || nch == 5 || nch == 8 || nch == 10 || nch == 12 || nch == 16)
                     : (nch == 2 || nch == 8);
}

hipError_t launch_b1_shape(clada_ctx *ctx, const B1Params &b, int Pb, int es, int nch, bool relu, bool dense,
                           bool *balance, hipStream_t stream)
{
    hipError_t eb = hipErrorNotSupported;
    for (int attempt = 0; attempt < 2 && eb == hipErrorNotSupported; ++attempt) {
        const bool bal = *balance;
        if (relu) {
            if (nch == 8) eb = launch_b1<2, 8, 16, true>(ctx, b, Pb, dense, bal, stream);
            else if (nch == 10) eb = launch_b1<2, 10, 8, true>(ctx, b, Pb, dense, bal, stream);
            else if (nch == 5) eb = launch_b1<2, 5, 16, true>(ctx, b, Pb, dense, bal, stream);
            else eb = launch_b1<2, 2, 16, true>(ctx, b, Pb, dense, bal, stream);
        }
        else if (es == 2 && nch == 8) eb = launch_b1<2, 8, 16>(ctx, b, Pb, dense, bal, stream);
        else if (es == 2 && nch == 10) eb = launch_b1<2, 10, 8>(ctx, b, Pb, dense, bal, stream);
        else if (es == 2 && nch == 12) eb = launch_b1<2, 12, 8>(ctx, b, Pb, dense, bal, stream);
        else if (es == 2 && nch == 16) eb = launch_b1<2, 16, 8>(ctx, b, Pb, dense, bal, stream);
        else if (es == 2 && nch == 5) eb = launch_b1<2, 5, 16>(ctx, b, Pb, dense, bal, stream);
        else if (es == 2 && nch == 4) eb = launch_b1<2, 4, 16>(ctx, b, Pb, dense, bal, stream);
        else if (es == 2 && nch == 2) eb = launch_b1<2, 2, 16>(ctx, b, Pb, dense, bal, stream);
        else if (es == 4 && nch == 2) eb = launch_b1<4, 2, 16>(ctx, b, Pb, dense, bal, stream);
        else if (es == 4 && nch == 8) eb = launch_b1<4, 8, 16>(ctx, b, Pb, dense, bal, stream);
        if (eb == hipErrorNotSupported) *balance = false;      // not co-resident: plain split-d
    }
    return eb;
}

// Balancing pays when the kept-row phase is long enough to hide the mask exchange behind the
// workgroup's own first chunk: measured faster on the 7B/8B shapes (90-117 MB per matrix), slower
// on 52 MB ReLU layers (17.0 vs 14.1 us) and on 8 MB ones (10.0 vs 6.4 us).  With 10 KiB gated rows
// (13B shape, own-first chunk of 7) it gains 2-3 % from sparsity 0.45 up and loses as much at 0.3.
bool b1_wants_balance(const clada_ctx *ctx, bool dense, bool relu, int ni_b, int d, int F, int es)
{
    const double phase2_bytes = (relu ? 1.0 : 2.0) * (double)F * d * es;
    return !dense && ni_b <= 56 && (ctx->opt_decode_b1 == 3 || (ctx->opt_decode_b1 == 1 && phase2_bytes >= 128e6));
}

template <int ES, int NCH, int NW, int GB, int UB>
hipError_t launch_decode(const DecodeParams &p, int P, int B, bool dense, hipStream_t st, bool list = false,
                         bool relu = false)
{
    constexpr int VEC = 16 / ES;
    const size_t lds = align_up(sizeof(int) * (3 * (size_t)p.ni_max + 4), 16) +
                       sizeof(float) * (size_t)(NW / 2) * NCH * 64 * VEC;
    auto kern = list ? (relu ? k_ffn_decode<ES, NCH, NW, GB, UB, true, true, true> : k_ffn_decode<ES, NCH, NW, GB, UB, true, true>)
                : relu ? (dense ? k_ffn_decode<ES, NCH, NW, GB, UB, true, false, true> : k_ffn_decode<ES, NCH, NW, GB, UB, false, false, true>)
                : dense ? k_ffn_decode<ES, NCH, NW, GB, UB, true> : k_ffn_decode<ES, NCH, NW, GB, UB, false>;
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
    p.keep = lists ? reinterpret_cast<unsigned char *>(ws + ws_partial_bytes(B, d)) : nullptr;
    p.idx = nullptr; p.n_list = nullptr; p.b_in = nullptr;
    p.gelu = layer->kind == CLADA_FFN_GEGLU ? 1 : 0;
    p.d = d; p.F = F; p.ni_max = (F + P - 1) / P;
    hipStream_t stream = (hipStream_t)hip_stream;

    const int nch = (d * es + 1023) / 1024;
    hipError_t e = hipErrorInvalidValue;

    const bool relu = layer->kind == CLADA_FFN_RELU;
    p.b_in = relu ? layer->b_in : nullptr;
    const float *b_out = relu ? layer->b_out : nullptr;

    // ---- split-d path (decode batch 1, whole-KiB rows, <= 64 neurons per workgroup)
    // (exactly the instantiations launched below: a shape admitted here without one would fail the call)
    const bool b1_shape = b1_shape_ok(es, nch, relu);
    if (ctx->opt_decode_b1 >= 1 && B == 1 && (d * es) % 1024 == 0 && b1_shape) {
        const int Pb = ctx->num_cu < COOP_MAX_WGS ? ctx->num_cu : COOP_MAX_WGS;
        const int ni_b = (F + Pb - 1) / Pb;
        if (F >= Pb && ni_b <= 1024) {
            B1Params b;
            b.wg = p.wg; b.wu = p.wu; b.wd = p.wd; b.x = p.x; b.tau = tau; b.partial = p.partial; b.keep = p.keep;
            b.rec = reinterpret_cast<unsigned long long *>(ctx->ws + COOP_REC);
            b.apub = reinterpret_cast<unsigned long long *>(ctx->ws + COOP_APUB);
            unsigned int *epoch = reinterpret_cast<unsigned int *>(ctx->ws + COOP_EPOCH);
            b.epoch = epoch;
            b.b_in = p.b_in;
            b.fault = reinterpret_cast<int *>(ctx->ws + COOP_FAULT);
            b.max_spins = ctx->opt_decode_spin_limit;
            b.d = d; b.F = F;
            b.K0 = ctx->opt_decode_own_first > 0 ? ctx->opt_decode_own_first : 14;
            b.gelu = p.gelu;
            bool balance = b1_wants_balance(ctx, dense, relu, ni_b, d, F, es);
            b.prev_partial = nullptr; b.prev_y = nullptr; b.prev_bias = nullptr; b.epoch_out = nullptr;
            hipError_t eb = launch_b1_shape(ctx, b, Pb, es, nch, relu, dense, &balance, stream);
            CLADA_CHECK_HIP(ctx, eb);
            launch_finalize(es, p.partial, Pb, 1, d, (char *)y, balance ? epoch : nullptr, stream,
                            ctx->opt_diag_events ? ctx->ev[2] : nullptr, ctx->ev[3], b_out, balance ? b.fault : nullptr);
            CLADA_CHECK_HIP(ctx, hipGetLastError());
            if (lists) {
                hipLaunchKernelGGL(k_ffn_lists, dim3(1), dim3(1024), 0, stream, p.keep, B, F, active_idx, n_active, mask_bits);
                CLADA_CHECK_HIP(ctx, hipGetLastError());
            }
            return CLADA_OK;
        }
    }
    // ---- batched MFMA path (bf16, supported widths): up to 16 tokens per pass; larger batches run
    // as ceil(B/16) passes of near-equal size, each re-reading the weights of its own union
    if (B >= 2 && ctx->opt_decode_batched) {
        unsigned char *keep_region = reinterpret_cast<unsigned char *>(ws + ws_partial_bytes(B, d));
        char *scratch = reinterpret_cast<char *>(keep_region) + align_up((size_t)B * F, 256);
        const int n_groups = (B + 15) / 16, per_group = (B + n_groups - 1) / n_groups;     // per_group >= 2 whenever B >= 2
        bool ran_all = false;
        if (ctx->opt_diag_events) CLADA_CHECK_HIP(ctx, hipEventRecord(ctx->ev[0], stream));
        for (int g0 = 0; g0 < B; g0 += per_group) {
            const int Bg = (B - g0 < per_group) ? B - g0 : per_group;
            bool ran = false;
            if (Bg >= 2)
                st = clada_decode_batched(ctx, layer, (const char *)x + (size_t)g0 * d * es, Bg, tau ? tau + g0 : nullptr,
                                          (char *)y + (size_t)g0 * d * es, p.keep ? p.keep + (size_t)g0 * F : nullptr,
                                          p.partial, scratch, dense, stream, &ran);
            if (st != CLADA_OK) return st;
            if (!ran) {
                // not eligible (decided by dtype and shape before anything is launched, so by the first
                // group) or a one-token remainder: the generic kernels below redo the whole batch
                ran_all = false;
                break;
            }
            ran_all = true;
        }
        if (ran_all) {
            if (ctx->opt_diag_events) {     // the batched path's final reduction is not timed apart
                CLADA_CHECK_HIP(ctx, hipEventRecord(ctx->ev[1], stream));
                CLADA_CHECK_HIP(ctx, hipEventRecord(ctx->ev[2], stream));
                CLADA_CHECK_HIP(ctx, hipEventRecord(ctx->ev[3], stream));
            }
            if (lists) {
                hipLaunchKernelGGL(k_ffn_lists, dim3(1), dim3(1024), 0, stream, p.keep, B, F, active_idx, n_active, mask_bits);
                CLADA_CHECK_HIP(ctx, hipGetLastError());
            }
            return CLADA_OK;
        }
    }
    if (ctx->opt_diag_events) CLADA_CHECK_HIP(ctx, hipEventRecord(ctx->ev[0], stream));
#define CLADA_DECODE_CASE(ES_, NCH_, NW_, GB_, UB_)                                        \
    if (es == ES_ && nch <= NCH_ && e == hipErrorInvalidValue)                             \
        e = launch_decode<ES_, NCH_, NW_, GB_, UB_>(p, P, B, dense, stream, false, relu);
    CLADA_DECODE_CASE(2, 1, 8, 2, 2)
    CLADA_DECODE_CASE(2, 2, 8, 2, 2)
    CLADA_DECODE_CASE(2, 4, 8, 2, 2)
    CLADA_DECODE_CASE(2, 8, 8, 1, 1)
    CLADA_DECODE_CASE(2, 10, 8, 1, 1)
    CLADA_DECODE_CASE(2, 16, 8, 1, 1)
    CLADA_DECODE_CASE(4, 1, 8, 2, 2)
    CLADA_DECODE_CASE(4, 2, 8, 2, 2)
    CLADA_DECODE_CASE(4, 4, 8, 2, 2)
    CLADA_DECODE_CASE(4, 8, 8, 1, 1)
    CLADA_DECODE_CASE(4, 16, 8, 1, 1)
#undef CLADA_DECODE_CASE
    CLADA_CHECK_HIP(ctx, e);

    if (ctx->opt_diag_events) CLADA_CHECK_HIP(ctx, hipEventRecord(ctx->ev[1], stream));
    launch_finalize(es, p.partial, P, B, d, (char *)y, nullptr, stream,
                    ctx->opt_diag_events ? ctx->ev[2] : nullptr, ctx->ev[3], b_out);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    if (lists) {
        hipLaunchKernelGGL(k_ffn_lists, dim3(1), dim3(1024), 0, stream, p.keep, B, F, active_idx, n_active, mask_bits);
        CLADA_CHECK_HIP(ctx, hipGetLastError());
    }
    return CLADA_OK;
}

// Decode over a caller-supplied neuron list (prefix-static masks): gate, up and down rows of the
// listed neurons only.
clada_status run_list_decode(clada_ctx *ctx, const clada_layer *layer, const void *x, int32_t B,
                             const int32_t *idx, const int32_t *n_active, void *y, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    clada_status st = clada_check_layer(ctx, layer);
    if (st != CLADA_OK) return st;
    if (!x || !y || !idx || !n_active) return clada_fail(ctx, CLADA_ERR_NULL, "x, y, active_idx or n_active is NULL");
    if (B < 1 || B > CLADA_MAX_BATCH) return clada_fail(ctx, CLADA_ERR_SHAPE, "B=%d outside [1,%d]", B, CLADA_MAX_BATCH);
    if (!aligned16(x) || !aligned16(y)) return clada_fail(ctx, CLADA_ERR_ALIGN, "x and y must be 16-byte aligned");
    const int d = layer->d, F = layer->d_ff;
    const size_t need = CLADA_WS_HEADER + clada_ws_decode(d, F, B);
    if (ctx->ws_bytes < need)
        return clada_fail(ctx, CLADA_ERR_WORKSPACE, "workspace %zu < %zu bytes needed", ctx->ws_bytes, need);
    const int es = (int)dtype_size(layer->dtype);
    int P = ctx->num_cu * ctx->opt_decode_wgs_per_cu;
    if (P > F) P = F;
    if (P > CLADA_MAX_DECODE_WGS) P = CLADA_MAX_DECODE_WGS;
    hipStream_t stream = (hipStream_t)hip_stream;
    DecodeParams p;
    p.wg = (const char *)layer->w_gate; p.wu = (const char *)layer->w_up; p.wd = (const char *)layer->w_down;
    p.x = (const char *)x; p.tau = nullptr;
    p.partial = reinterpret_cast<float *>(ctx->ws + CLADA_WS_HEADER);
    p.keep = nullptr; p.idx = idx; p.n_list = n_active;
    p.d = d; p.F = F; p.ni_max = (F + P - 1) / P;
    p.gelu = layer->kind == CLADA_FFN_GEGLU ? 1 : 0;
    const bool relu = layer->kind == CLADA_FFN_RELU;
    p.b_in = relu ? layer->b_in : nullptr;
    const float *b_out = relu ? layer->b_out : nullptr;
    const int nch = (d * es + 1023) / 1024;
    // ---- matrix-core path (bf16, supported widths), up to 16 tokens per pass, as in the thresholded call
    if (B >= 2 && ctx->opt_decode_batched) {
        char *ws = ctx->ws + CLADA_WS_HEADER;
        char *scratch = ws + ws_partial_bytes(B, d) + align_up((size_t)B * F, 256);
        const int n_groups = (B + 15) / 16, per_group = (B + n_groups - 1) / n_groups;
        bool ran_all = false;
        for (int g0 = 0; g0 < B; g0 += per_group) {
            const int Bg = (B - g0 < per_group) ? B - g0 : per_group;
            bool ran = false;
            if (Bg >= 2) {
                st = clada_decode_batched(ctx, layer, (const char *)x + (size_t)g0 * d * es, Bg, nullptr,
                                          (char *)y + (size_t)g0 * d * es, nullptr, p.partial, scratch, true, stream, &ran,
                                          idx, n_active);
                if (st != CLADA_OK) return st;
            }
            ran_all = ran;
            if (!ran) break;                                // not eligible, or a one-token remainder: generic kernels redo the batch
        }
        if (ran_all) return CLADA_OK;
    }
    if (B == 1 && ctx->opt_decode_b1 >= 1) {            // streaming kernel for whole-KiB rows
        bool ran = false;
        int Pl = 0;
        CLADA_CHECK_HIP(ctx, clada_decode_list_b1(ctx, layer, x, idx, n_active, p.partial, &Pl, stream, &ran));
        if (ran) {
            launch_finalize(es, p.partial, Pl, 1, d, (char *)y, nullptr, stream, nullptr, nullptr, b_out);
            CLADA_CHECK_HIP(ctx, hipGetLastError());
            return CLADA_OK;
        }
    }
    hipError_t e = hipErrorInvalidValue;
#define CLADA_LIST_CASE(ES_, NCH_, NW_, GB_, UB_)                                          \
    if (es == ES_ && nch <= NCH_ && e == hipErrorInvalidValue)                             \
        e = launch_decode<ES_, NCH_, NW_, GB_, UB_>(p, P, B, true, stream, true, relu);
    CLADA_LIST_CASE(2, 1, 8, 2, 2)
    CLADA_LIST_CASE(2, 2, 8, 2, 2)
    CLADA_LIST_CASE(2, 4, 8, 2, 2)
    CLADA_LIST_CASE(2, 8, 8, 1, 1)
    CLADA_LIST_CASE(2, 10, 8, 1, 1)
    CLADA_LIST_CASE(2, 16, 8, 1, 1)
    CLADA_LIST_CASE(4, 1, 8, 2, 2)
    CLADA_LIST_CASE(4, 2, 8, 2, 2)
    CLADA_LIST_CASE(4, 4, 8, 2, 2)
    CLADA_LIST_CASE(4, 8, 8, 1, 1)
    CLADA_LIST_CASE(4, 16, 8, 1, 1)
#undef CLADA_LIST_CASE
    CLADA_CHECK_HIP(ctx, e);
    launch_finalize(es, p.partial, P, B, d, (char *)y, nullptr, stream, nullptr, nullptr, b_out);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    return CLADA_OK;
}

// ---- whole-stack entry points (B = 1)
template <int ES, int NCH, int DCH, bool DENSE, bool BAL, bool RELU>
hipError_t launch_stack_variant(clada_ctx *ctx, const StackParams &p, int P, hipStream_t st)
{
    auto kern = k_ffn_decode_b1<ES, NCH, 8, DCH, DENSE, BAL, RELU, true>;
    // every workgroup waits for the others' partials (and masks): all of them must be resident at once
    const void *fn = reinterpret_cast<const void *>(kern);
    int occ = -1;
    for (int i = 0; i < ctx->n_occ; ++i)
        if (ctx->occ_fn[i] == fn) occ = ctx->occ_val[i];
    if (occ < 0) {
        int nb = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, 512, 0);
        if (e != hipSuccess) return e;
        occ = nb;
        if (ctx->n_occ < CLADA_OCC_SLOTS) {
            ctx->occ_fn[ctx->n_occ] = fn;
            ctx->occ_val[ctx->n_occ++] = nb;
        }
    }
    if ((long long)occ * ctx->num_cu < P) return hipErrorNotSupported;
    hipLaunchKernelGGL(kern, dim3(P), dim3(512), 0, st, p);
    return hipGetLastError();
}

template <int ES, int NCH, int DCH, bool RELU = false>
hipError_t launch_stack(clada_ctx *ctx, const StackParams &p, int P, bool dense, bool balance, hipStream_t st)
{
    if (dense) return launch_stack_variant<ES, NCH, DCH, true, false, RELU>(ctx, p, P, st);
    if (balance) return launch_stack_variant<ES, NCH, DCH, false, true, RELU>(ctx, p, P, st);
    return launch_stack_variant<ES, NCH, DCH, false, false, RELU>(ctx, p, P, st);
}

// Lanes of the whole-stack calls: lane 0 is the caller's stream, the others belong to the context.  lanes_fork
// makes the further lanes wait for what the caller's stream holds so far, lanes_join makes the caller's stream
// wait for them; both are events, so a capture of the caller's stream takes the lanes in.
hipError_t lanes_fork(clada_ctx *ctx, int n_lanes, hipStream_t stream)
{
    if (n_lanes < 2) return hipSuccess;
    hipError_t e;
    for (int i = 0; i < n_lanes - 1; ++i)
        if (!ctx->lane_stream[i] && (e = hipStreamCreateWithFlags(&ctx->lane_stream[i], hipStreamNonBlocking)) != hipSuccess) return e;
    for (int i = 0; i < 4; ++i)
        if (!ctx->ev_lane[i] && (e = hipEventCreateWithFlags(&ctx->ev_lane[i], hipEventDisableTiming)) != hipSuccess) return e;
    if ((e = hipEventRecord(ctx->ev_lane[0], stream)) != hipSuccess) return e;
    for (int i = 0; i < n_lanes - 1; ++i)
        if ((e = hipStreamWaitEvent(ctx->lane_stream[i], ctx->ev_lane[0], 0)) != hipSuccess) return e;
    return hipSuccess;
}

hipError_t lanes_join(clada_ctx *ctx, int n_lanes, hipStream_t stream)
{
    hipError_t e;
    for (int i = 0; i < n_lanes - 1; ++i) {
        if ((e = hipEventRecord(ctx->ev_lane[1 + i], ctx->lane_stream[i])) != hipSuccess) return e;
        if ((e = hipStreamWaitEvent(stream, ctx->ev_lane[1 + i], 0)) != hipSuccess) return e;
    }
    return hipSuccess;
}

// Scratch of lane 1 and 2 for batches (lane 0 uses the regions of the per-layer call): partial outputs of one
// pass and the batched path's own scratch, behind everything else of the decode workspace.
size_t ws_lane_bytes(int d, int F) { return clada_ws_decode_batched_partial(d) + clada_ws_decode_batched(F); }

clada_status run_stack_decode(clada_ctx *ctx, const clada_layer *layers, int32_t L, const void *x, int32_t B,
                              const float *tau, void *y, int32_t *n_active, bool dense, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    if (!layers) return clada_fail(ctx, CLADA_ERR_NULL, "layers is NULL");
    if (L < 1 || L > CLADA_MAX_LAYERS) return clada_fail(ctx, CLADA_ERR_SHAPE, "L=%d outside [1,%d]", L, CLADA_MAX_LAYERS);
    for (int l = 0; l < L; ++l) {
        clada_status st = clada_check_layer(ctx, &layers[l]);
        if (st != CLADA_OK) return st;
        if (layers[l].d != layers[0].d || layers[l].d_ff != layers[0].d_ff || layers[l].dtype != layers[0].dtype ||
            layers[l].kind != layers[0].kind)
            return clada_fail(ctx, CLADA_ERR_SHAPE, "layer %d differs from layer 0 in d, d_ff, dtype or kind", l);
    }
    if (!x || !y || (!dense && !tau)) return clada_fail(ctx, CLADA_ERR_NULL, "x, y or tau_final is NULL");
    if (B < 1 || B > CLADA_MAX_BATCH) return clada_fail(ctx, CLADA_ERR_SHAPE, "B=%d outside [1,%d]", B, CLADA_MAX_BATCH);
    if (!aligned16(x) || !aligned16(y)) return clada_fail(ctx, CLADA_ERR_ALIGN, "x and y must be 16-byte aligned");
    const int d = layers[0].d, F = layers[0].d_ff;
    const size_t need = CLADA_WS_HEADER + clada_ws_decode(d, F, B);
    if (ctx->ws_bytes < need)
        return clada_fail(ctx, CLADA_ERR_WORKSPACE, "workspace %zu < %zu bytes needed", ctx->ws_bytes, need);
    const int es = (int)dtype_size(layers[0].dtype);
    const int nch = (d * es + 1023) / 1024;
    const bool relu = layers[0].kind == CLADA_FFN_RELU;
    hipStream_t stream = (hipStream_t)hip_stream;
    const int Pb = ctx->num_cu < COOP_MAX_WGS ? ctx->num_cu : COOP_MAX_WGS;
    const int ni_b = Pb > 0 ? (F + Pb - 1) / Pb : 0;
    // shapes the persistent kernel is built for (the widths of the models the paper evaluates); anything
    // else, and a launch that cannot hold all its workgroups at once, runs as L per-layer calls
    const bool shape_ok = (d * es) % 1024 == 0 && es == 2 &&
                          (relu ? nch == 5 : (nch == 4 || nch == 8 || nch == 10));
    bool persistent = B == 1 && ctx->opt_decode_stack == 1 && ctx->opt_decode_b1 >= 1 && shape_ok && F >= Pb && ni_b <= 64;
    if (persistent) {
        const double phase2_bytes = (relu ? 1.0 : 2.0) * (double)F * d * es;
        const bool balance = !dense && ni_b <= 56 &&
                             (ctx->opt_decode_b1 == 3 || (ctx->opt_decode_b1 == 1 && phase2_bytes >= 128e6));
        for (int l0 = 0; l0 < L && persistent; l0 += CLADA_STACK_MAX_LAYERS) {
            const int n = L - l0 < CLADA_STACK_MAX_LAYERS ? L - l0 : CLADA_STACK_MAX_LAYERS;
            StackParams sp;
            memset(&sp, 0, sizeof(sp));
            for (int l = 0; l < n; ++l) {
                sp.wg[l] = (const char *)layers[l0 + l].w_gate;
                sp.wu[l] = (const char *)layers[l0 + l].w_up;
                sp.wd[l] = (const char *)layers[l0 + l].w_down;
                sp.b_in[l] = relu ? layers[l0 + l].b_in : nullptr;
                sp.b_out[l] = relu ? layers[l0 + l].b_out : nullptr;
            }
            sp.x = (const char *)x + (size_t)l0 * d * es;
            sp.y = (char *)y + (size_t)l0 * d * es;
            sp.tau = tau ? tau + l0 : nullptr;
            sp.partial = reinterpret_cast<float *>(ctx->ws + CLADA_WS_HEADER);
            sp.rec = reinterpret_cast<unsigned long long *>(ctx->ws + STACK_REC);
            sp.apub = reinterpret_cast<unsigned long long *>(ctx->ws + STACK_APUB);
            sp.epoch = reinterpret_cast<unsigned int *>(ctx->ws + STACK_EPOCH);
            sp.kcnt = reinterpret_cast<int *>(ctx->ws + STACK_KCNT);
            sp.n_active = (n_active && !dense) ? n_active + 2 * l0 : nullptr;
            sp.fault = reinterpret_cast<int *>(ctx->ws + COOP_FAULT);
            sp.max_spins = ctx->opt_decode_spin_limit;
            sp.d = d; sp.F = F; sp.L = n;
            sp.K0 = ctx->opt_decode_own_first > 0 ? ctx->opt_decode_own_first : 14;
            sp.gelu = layers[0].kind == CLADA_FFN_GEGLU ? 1 : 0;
            hipError_t e = hipErrorNotSupported;
            if (relu) e = launch_stack<2, 5, 16, true>(ctx, sp, Pb, dense, balance, stream);
            else if (nch == 8) e = launch_stack<2, 8, 16>(ctx, sp, Pb, dense, balance, stream);
            else if (nch == 10) e = launch_stack<2, 10, 8>(ctx, sp, Pb, dense, balance, stream);
            else if (nch == 4) e = launch_stack<2, 4, 16>(ctx, sp, Pb, dense, balance, stream);
            if (e == hipErrorNotSupported && l0 == 0) { persistent = false; break; }
            CLADA_CHECK_HIP(ctx, e);
        }
        if (persistent) return CLADA_OK;
    }
    // ---- launches issued by the library itself.  Two things the per-layer calls cannot do:
    // * lanes (the default): the layers of a stack are independent problems, so they go round two or three
    //   HIP streams (the caller's and the context's own, forked and joined by events, which a stream
    //   capture follows).  A compute unit that has finished its share of layer l takes a workgroup of
    //   layer l+1 at once: the start-up and the ragged end of every kernel are covered by its neighbour
    //   (7B layer shape, sparsity 0.45: 36.0 -> 32.5 us per layer; three and four lanes are slower again).
    //   Kernels that wait for each other's workgroups must not share the chip, so the lanes run the
    //   unbalanced instances.
    // * chained launches (one lane): a layer's kernel also sums the partial outputs of the previous layer,
    //   which a kernel boundary has made complete and visible, so only the last layer needs a reduction
    //   launch; the partials alternate between two buffers (36.0 -> 35.1 us per layer; inside two lanes the
    //   reduction launches are covered anyway and chaining loses 0.6 us).
    // Counts per layer need the flag arrays and the list kernel of the per-layer call, so a call that asks
    // for them runs the per-layer calls below.
    const int smode = ctx->opt_decode_stack;
    const bool own_launches = B == 1 && smode >= 2 && ctx->opt_decode_b1 >= 1 && !n_active && (d * es) % 1024 == 0 &&
                              b1_shape_ok(es, nch, relu) && Pb == COOP_MAX_WGS && F >= Pb && ni_b <= 1024 && L >= 2;
    if (own_launches) {
        static_assert(COOP_MAX_WGS == 256, "the chained reduction is laid out for 256 partial outputs");
        // Rows of 4, 5 and 8 KiB have an instance of which two workgroups fit a compute unit: with it, workgroups
        // of different layers share every unit (measured, 7B shape, ms per step of 32 layers at sparsity 0.45 /
        // dense: two lanes 1.038 / 1.379 with the one-per-unit instance, 1.031 / 1.330 with this one; three lanes
        // 1.085 / 1.460 and 1.006 / 1.357; four lanes 1.041 / 1.391 with this one)
        const bool occ2 = b1_occ2_shape_ok(es, nch, relu) && ni_b <= 64 && ctx->opt_decode_lane_occ2 != 0;
        const int n_lanes = (smode == 3 && L >= 4) ? ((occ2 && !dense) ? 3 : 2) : 1;
        const bool chained = smode == 2;
        unsigned int *epoch = reinterpret_cast<unsigned int *>(ctx->ws + COOP_EPOCH);
        float *part = reinterpret_cast<float *>(ctx->ws + CLADA_WS_HEADER);
        bool balance = smode == 2 && b1_wants_balance(ctx, dense, relu, ni_b, d, F, es);      // (mode 3 never balances, whatever L: one set of bits)
        B1Params b;
        b.keep = nullptr;
        b.rec = reinterpret_cast<unsigned long long *>(ctx->ws + COOP_REC);
        b.apub = reinterpret_cast<unsigned long long *>(ctx->ws + COOP_APUB);
        b.epoch = epoch;
        b.fault = reinterpret_cast<int *>(ctx->ws + COOP_FAULT);
        b.max_spins = ctx->opt_decode_spin_limit;
        b.d = d; b.F = F;
        b.K0 = ctx->opt_decode_own_first > 0 ? ctx->opt_decode_own_first : 14;
        b.gelu = layers[0].kind == CLADA_FFN_GEGLU ? 1 : 0;
        CLADA_CHECK_HIP(ctx, lanes_fork(ctx, n_lanes, stream));
        const size_t buf = (size_t)Pb * d;                   // floats of one buffer of partial outputs
        for (int l = 0; l < L; ++l) {
            const int lane = l % n_lanes, k = l / n_lanes;   // the layer is its lane's k-th
            hipStream_t st = lane ? ctx->lane_stream[lane - 1] : stream;
            float *mine = part + (size_t)(chained ? 2 * lane + (k & 1) : lane) * buf;
            const int lp = l - n_lanes;                      // the lane's previous layer
            b.wg = (const char *)layers[l].w_gate; b.wu = (const char *)layers[l].w_up; b.wd = (const char *)layers[l].w_down;
            b.b_in = relu ? layers[l].b_in : nullptr;
            b.x = (const char *)x + (size_t)l * d * es;
            b.tau = tau ? tau + l : nullptr;
            b.partial = mine;
            const bool sums_prev = chained && lp >= 0;
            b.prev_partial = sums_prev ? part + (size_t)(2 * lane + ((k - 1) & 1)) * buf : nullptr;      // (chained: one lane)
            b.prev_y = sums_prev ? (char *)y + (size_t)lp * d * es : nullptr;
            b.prev_bias = (sums_prev && relu) ? layers[lp].b_out : nullptr;
            b.epoch_out = epoch;                             // only the balanced instance writes it
            if (n_lanes >= 2 && occ2)
                CLADA_CHECK_HIP(ctx, launch_b1_occ2(b, Pb, nch, relu, dense, st));
            else
                CLADA_CHECK_HIP(ctx, launch_b1_shape(ctx, b, Pb, es, nch, relu, dense, &balance, st));
            if (!chained || l + n_lanes >= L) {              // nobody after it in its lane: its own reduction launch
                launch_finalize(es, mine, Pb, 1, d, (char *)y + (size_t)l * d * es, (!chained && balance) ? epoch : nullptr, st,
                                nullptr, nullptr, relu ? layers[l].b_out : nullptr, balance ? b.fault : nullptr);
                CLADA_CHECK_HIP(ctx, hipGetLastError());
            }
        }
        CLADA_CHECK_HIP(ctx, lanes_join(ctx, n_lanes, stream));
        return CLADA_OK;
    }
    // ---- batches on the matrix-core path: the units (layer, pass of up to 16 tokens) go round three lanes, each
    // with its own partial outputs and scratch.  The path's three launches per unit and its thin ends weigh
    // more than at batch 1 (c3 layer shape, B = 8: 69.5 -> 60.2 -> 58.5 us per layer with one, two, three lanes).
    const int n_groups = (B + 15) / 16, per_group = (B + n_groups - 1) / n_groups;
    if (B >= 2 && smode == 3 && !n_active && ctx->opt_decode_batched && L * n_groups >= 3 &&
        clada_decode_batched_eligible(ctx, &layers[0], per_group) &&
        clada_decode_batched_eligible(ctx, &layers[0], B - (n_groups - 1) * per_group)) {
        const int n_lanes = 3;
        char *ws = ctx->ws + CLADA_WS_HEADER;
        char *lane_base[3];
        lane_base[0] = nullptr;
        lane_base[1] = ws + clada_ws_decode(d, F, B) - 2 * ws_lane_bytes(d, F);
        lane_base[2] = lane_base[1] + ws_lane_bytes(d, F);
        CLADA_CHECK_HIP(ctx, lanes_fork(ctx, n_lanes, stream));
        int unit = 0;
        for (int l = 0; l < L; ++l)
            for (int g0 = 0; g0 < B; g0 += per_group, ++unit) {
                const int Bg = (B - g0 < per_group) ? B - g0 : per_group;
                const int lane = unit % n_lanes;
                float *partial = lane ? reinterpret_cast<float *>(lane_base[lane]) : reinterpret_cast<float *>(ws);
                char *scratch = lane ? lane_base[lane] + clada_ws_decode_batched_partial(d)
                                     : ws + ws_partial_bytes(B, d) + align_up((size_t)B * F, 256);
                const size_t row = (size_t)l * B + g0;
                bool ran = false;
                clada_status st = clada_decode_batched(ctx, &layers[l], (const char *)x + row * d * es, Bg, tau ? tau + row : nullptr,
                                                       (char *)y + row * d * es, nullptr, partial, scratch, dense,
                                                       lane ? ctx->lane_stream[lane - 1] : stream, &ran);
                if (st != CLADA_OK || !ran) {
                    (void)lanes_join(ctx, n_lanes, stream);      // leave no lane forked (a capture would not end)
                    return st != CLADA_OK ? st : clada_fail(ctx, CLADA_ERR_SHAPE, "batched path refused a unit it had accepted");
                }
            }
        CLADA_CHECK_HIP(ctx, lanes_join(ctx, n_lanes, stream));
        return CLADA_OK;
    }
    for (int l = 0; l < L; ++l) {
        const size_t row = (size_t)l * B;
        clada_status st = run_decode(ctx, &layers[l], (const char *)x + row * d * es, B, tau ? tau + row : nullptr,
                                     (char *)y + row * d * es, nullptr, n_active ? n_active + (size_t)(1 + B) * l : nullptr,
                                     nullptr, dense, hip_stream);
        if (st != CLADA_OK) return st;
    }
    return CLADA_OK;
}

}  // namespace

extern "C" clada_status clada_static_ffn_decode(clada_ctx *ctx, const clada_layer *layer, const void *x,
                                                int32_t B, const int32_t *active_idx, const int32_t *n_active,
                                                void *y, void *hip_stream)
{
    return run_list_decode(ctx, layer, x, B, active_idx, n_active, y, hip_stream);
}

void clada_launch_finalize(int es, const float *partial, int P, int B, int d, char *y, hipStream_t stream,
                           const float *bias)
{
    launch_finalize(es, partial, P, B, d, y, nullptr, stream, nullptr, nullptr, bias);
}

size_t clada_ws_decode(int32_t d, int32_t d_ff, int32_t B)
{
    if (B <= 0) return 0;
    return ws_partial_bytes(B, d) + align_up((size_t)B * d_ff, 256) +
           clada_ws_decode_batched(d_ff) + (B >= 2 ? 2 * ws_lane_bytes(d, d_ff) : 0);
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

extern "C" clada_status clada_sparse_ffn_stack_decode(clada_ctx *ctx, const clada_layer *layers, int32_t L,
                                                      const void *x, int32_t B, const float *tau_final, void *y,
                                                      int32_t *n_active, void *hip_stream)
{
    return run_stack_decode(ctx, layers, L, x, B, tau_final, y, n_active, false, hip_stream);
}

extern "C" clada_status clada_dense_ffn_stack_decode(clada_ctx *ctx, const clada_layer *layers, int32_t L,
                                                     const void *x, int32_t B, void *y, void *hip_stream)
{
    return run_stack_decode(ctx, layers, L, x, B, nullptr, y, nullptr, true, hip_stream);
}
