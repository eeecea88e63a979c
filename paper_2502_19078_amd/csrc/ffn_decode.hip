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

// y[b][col] = sum_p partial[p][b][col].  A workgroup owns 32 columns; thread (slice, colgroup)
// adds the partials p = slice, slice+32, ... (all loads issued together), the 32 slices are
// folded by a fixed tree; one rounding to the output dtype.
template <int ES>
__global__ void __launch_bounds__(256)
k_ffn_finalize(const float *__restrict__ partial, int P, int d, char *__restrict__ y, unsigned int *epoch)
{
    if (epoch && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *epoch += 1u;   // cooperative call counter
    __shared__ float4 s_sum[32][8];
    const int cg = threadIdx.x & 7, sl = threadIdx.x >> 3;
    const int col = blockIdx.x * 32 + cg * 4;
    const int b = blockIdx.y, B = gridDim.y;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (col < d) {
        const float *base = partial + (size_t)b * d + col;
        const size_t pstride = (size_t)B * d;
        int q = sl;
        for (; q + 7 * 32 < P; q += 8 * 32) {
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4 *>(base + (size_t)(q + u * 32) * pstride);
#pragma unroll
            for (int u = 0; u < 8; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
        }
        for (; q < P; q += 32) {
            const float4 v = *reinterpret_cast<const float4 *>(base + (size_t)q * pstride);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
    }
    s_sum[sl][cg] = s;
    __syncthreads();
#pragma unroll
    for (int h = 16; h >= 1; h >>= 1) {
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

void launch_finalize(int es, const float *partial, int P, int B, int d, char *y, unsigned int *epoch, hipStream_t stream)
{
    const dim3 grid((d + 31) / 32, B);
    if (es == 4) hipLaunchKernelGGL(k_ffn_finalize<4>, grid, dim3(256), 0, stream, partial, P, d, y, epoch);
    else         hipLaunchKernelGGL(k_ffn_finalize<2>, grid, dim3(256), 0, stream, partial, P, d, y, epoch);
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


// ---------------------------------------------------------------------------------------
// Cooperative single-kernel path for decode batch 1 (the configuration the method is
// timed on).  Same gate / compaction / up-down structure as k_ffn_decode, plus:
//   * load balancing: a workgroup's kept count is binomial, so with a static neuron split
//     the slowest workgroup would set the kernel time.  Each workgroup publishes its keep
//     mask (<= 56 neurons -> one 64-bit word, tagged with the call's epoch) and its
//     activations, processes its own first K0 kept neurons, then reads all P masks and
//     takes its share of the pooled surplus so that every workgroup handles floor/ceil(k/P)
//     neurons.  The assignment is a function of the masks only, so the summation order --
//     and the result -- stays bit-reproducible.
//   * the cross-workgroup reduction of the partial y's runs in the same kernel: after
//     publishing its partial every workgroup waits for all P "done" tags and adds its own
//     slice of columns over the partials in fixed order (no separate finalize launch).
// All P workgroups must be co-resident (checked on the host: P <= CUs * occupancy).
// Cross-workgroup data goes through agent-scope release stores / acquire loads.
struct CoopParams {
    const char *wg, *wu, *wd, *x;
    const float *tau;
    char *y;
    unsigned long long *rec;    // [P] keep mask of the workgroup's neurons (bit i = neuron blk + P*i,
                                //     i < 56) | 8-bit epoch tag in bits 56..63, stored with release
    float *apub;                // [P][64] published activations a_i of the workgroup's neurons
    float *partial;             // [P][d]
    const unsigned int *epoch;  // device-side call counter (survives graph replays); advanced by k_ffn_finalize
    unsigned char *keep;        // [F] or nullptr
    int d, F, K0;
};

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

__device__ __forceinline__ int block_excl_scan(int v, int tid, int *s_tmp, int nwaves, int *total)
{   // exclusive prefix sum over the workgroup's threads (all threads must call)
    const int lane = tid & 63, wave = tid >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    if (lane == 63) s_tmp[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
    for (int w = 0; w < nwaves; ++w) {
        const int c = s_tmp[w];
        if (w < wave) base += c;
        tot += c;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

template <int ES, int NCH, int NW, bool DENSE>
__global__ void __launch_bounds__(NW * 64)
k_ffn_decode_coop(const CoopParams p)
{
    constexpr int VEC = 16 / ES;
    constexpr int ROWB = NCH * 1024;                       // full rows only: d*ES == NCH*1024
    __shared__ float s_a[64];
    __shared__ int s_flag[64];
    __shared__ int s_list[64];
    __shared__ int s_l2row[64];
    __shared__ int s_l2a[64];
    __shared__ int s_tmp[NW];
    __shared__ int s_misc[4];
    extern __shared__ __align__(16) unsigned char smem_coop[];
    float *s_red = reinterpret_cast<float *>(smem_coop);   // fold buffers, later the reduction staging

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int blk = blockIdx.x, P = gridDim.x;
    const int F = p.F;
    const int ni = blk < F ? (F - blk + P - 1) / P : 0;    // <= 56
    // Every cooperative call (sparse or dense) rewrites all P records, so a stale record is
    // exactly one call old and an 8-bit tag tells it apart.
    const unsigned int ep = *p.epoch + 1u;
    const unsigned long long tag = (unsigned long long)(ep & 0xffu) << 56;
    const int loff = lane * 16;

    float xr[NCH][VEC];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
        unpack_row16(*reinterpret_cast<const u32x4 *>(p.x + c * 1024 + loff), xr[c]);
    const float tau = DENSE ? 0.0f : p.tau[0];

    // ---------------------------------------------------------------- gate phase
    for (int i = wave; i < ni; i += NW) {
        const char *row = p.wg + (size_t)(blk + P * i) * ROWB + loff;
        u32x4 buf[NCH];
#pragma unroll
        for (int c = 0; c < NCH; ++c) buf[c] = ld_stream16(row + c * 1024);
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            float w[VEC];
            unpack_row16(buf[c], w);
#pragma unroll
            for (int e = 0; e < VEC; ++e) s = fmaf(w[e], xr[c][e], s);
        }
        s = wave_sum(s);
        const float a = silu_f32(s);
        const bool keep = DENSE ? true : (fabsf(a) >= tau);
        if (lane == 0) {
            s_a[i] = a;
            s_flag[i] = keep ? 1 : 0;
            if (p.keep) p.keep[blk + P * i] = keep ? 1 : 0;
        }
    }
    __syncthreads();

    // every wave derives the same mask and list (no second barrier needed)
    const unsigned long long mask = __ballot(lane < ni && s_flag[lane] != 0);
    const int kp = __popcll(mask);
    if ((mask >> lane) & 1ull) s_list[__popcll(mask & ((1ull << lane) - 1ull))] = lane;
    const int own = DENSE ? kp : min(kp, p.K0);
    if (wave == 0) {
        // Publish activations, then the tagged mask.  Both go out as agent-scope atomic stores
        // (written through to memory), so ordering them needs only the wait for the first
        // stores' acknowledgements (a workgroup-scope release fence), not an L2 write-back.
        if (!DENSE && lane < ni)
            __hip_atomic_store(p.apub + blk * 64 + lane, s_a[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (lane == 0) __hip_atomic_store(p.rec + blk, mask | tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    float acc[NCH][VEC];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[c][e] = 0.0f;

    auto updown = [&](int row_j, float a, const float *a_pub) {
        const size_t off = (size_t)row_j * ROWB + loff;
        u32x4 ub[NCH], db[NCH];
        // a borrowed neuron's activation travels with its weight rows (same round trip)
        if (a_pub) a = __hip_atomic_load(a_pub, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int c = 0; c < NCH; ++c) ub[c] = ld_stream16(p.wu + off + c * 1024);
#pragma unroll
        for (int c = 0; c < NCH; ++c) db[c] = ld_stream16(p.wd + off + c * 1024);
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            float w[VEC];
            unpack_row16(ub[c], w);
#pragma unroll
            for (int e = 0; e < VEC; ++e) s = fmaf(w[e], xr[c][e], s);
        }
        const float h = a * wave_sum(s);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            float w[VEC];
            unpack_row16(db[c], w);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[c][e] = fmaf(h, w[e], acc[c][e]);
        }
    };

    // ------------------------------------------- own kept neurons (first `own` of the list)
    for (int t = wave; t < own; t += NW) {
        const int i = s_list[t];
        updown(blk + P * i, s_a[i], nullptr);
    }

    // ------------------------------------------- share of the pooled surplus
    int n2 = 0;
    if (!DENSE) {
        // thread q polls record q (relaxed loads that go to memory, spaced by s_sleep); all cross-
        // workgroup reads below are agent-scope atomic loads, so no cache invalidation is needed
        unsigned long long mq = 0ull;
        if (tid < P) {
            for (;;) {
                mq = __hip_atomic_load(p.rec + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((mq & (0xffull << 56)) == tag) break;
                __builtin_amdgcn_s_sleep(8);
            }
            mq &= ~(0xffull << 56);
        }
        const int kq = __popcll(mq);
        const int oq = min(kq, p.K0), sq = kq - oq;
        int K, S;
        (void)block_excl_scan(kq, tid, s_tmp, NW, &K);
        // target count of workgroup q: floor((q+1)K/P) - floor(qK/P); extra beyond its own first rows
        const int tgt = tid < P ? (int)(((long long)(tid + 1) * K) / P - ((long long)tid * K) / P) : 0;
        const int eq = max(0, tgt - oq);
        // one scan for both prefixes: surplus counts in the low half, extras in the high half
        int SE;
        const int sepre = block_excl_scan(sq | (eq << 16), tid, s_tmp, NW, &SE);
        const int spre = sepre & 0xffff, epre = sepre >> 16;
        S = SE & 0xffff;
        if (tid == blk) {
            s_misc[0] = min(epre, S);
            s_misc[1] = min(epre + eq, S);
        }
        __syncthreads();
        const int lo = s_misc[0], hi = s_misc[1];
        n2 = hi - lo;
        // thread q hands over the part of its surplus [spre, spre+sq) that falls into [lo, hi)
        const int a0 = max(lo, spre), a1 = min(hi, spre + sq);
        for (int r = a0; r < a1; ++r) {
            const int i = select_bit(mq, oq + (r - spre));
            s_l2row[r - lo] = tid + P * i;
            s_l2a[r - lo] = tid * 64 + i;
        }
        __syncthreads();
        const int shift = own % NW;                         // wave that would take list entry `own`
        for (int r = (wave - shift + NW) % NW; r < n2; r += NW) updown(s_l2row[r], 0.0f, p.apub + s_l2a[r]);
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
        float *dst = p.partial + (size_t)blk * p.d;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int e = 0; e < VEC; e += 4)
                *reinterpret_cast<float4 *>(dst + (c * 64 + lane) * VEC + e) =
                    make_float4(acc[c][e], acc[c][e + 1], acc[c][e + 2], acc[c][e + 3]);
    }
    // the epoch is advanced by the finalize kernel that follows on the stream
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

// Cooperative launch; returns hipErrorNotSupported when the shape is not eligible.
template <int ES, int NCH>
hipError_t launch_coop(clada_ctx *ctx, const CoopParams &p, int P, bool dense, hipStream_t st)
{
    constexpr int NW = 8, VEC = 16 / ES;
    const size_t lds = sizeof(float) * (size_t)(NW / 2) * NCH * 64 * VEC;
    auto kern = dense ? k_ffn_decode_coop<ES, NCH, NW, true> : k_ffn_decode_coop<ES, NCH, NW, false>;
    static int occ_cache[2] = {-1, -1};                    // per instantiation (template statics)
    if (occ_cache[dense] < 0) {
        hipError_t e = hipSuccess;
        if (lds > 48 * 1024)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        int nb = 0;
        if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, NW * 64, lds);
        if (e != hipSuccess) return e;
        occ_cache[dense] = nb;
    }
    if ((long long)occ_cache[dense] * ctx->num_cu < P) return hipErrorNotSupported;   // not co-resident
    hipLaunchKernelGGL(kern, dim3(P), dim3(NW * 64), lds, st, p);
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

    // ---- cooperative single-kernel path (decode batch 1, whole-KiB rows, <= 56 neurons per workgroup)
    if (ctx->opt_decode_coop && B == 1 && (d * es) % 1024 == 0 && (nch == 2 || nch == 8 || nch == 10)) {
        // the record tags rely on every cooperative call using the same P
        const int Pc = ctx->num_cu < COOP_MAX_WGS ? ctx->num_cu : COOP_MAX_WGS;
        const int ni_c = (F + Pc - 1) / Pc;
        if (F >= Pc && ni_c <= 56) {
            CoopParams c;
            c.wg = p.wg; c.wu = p.wu; c.wd = p.wd; c.x = p.x; c.tau = tau; c.y = (char *)y;
            c.rec = reinterpret_cast<unsigned long long *>(ctx->ws + COOP_REC);
            c.apub = reinterpret_cast<float *>(ctx->ws + COOP_APUB);
            c.partial = p.partial;
            c.epoch = reinterpret_cast<unsigned int *>(ctx->ws + COOP_EPOCH);
            c.keep = p.keep;
            c.d = d; c.F = F;
            c.K0 = ctx->opt_decode_own_first > 0 ? ctx->opt_decode_own_first : (ni_c / 3 > 1 ? ni_c / 3 : 1);
            hipError_t ec = hipErrorNotSupported;
            if (es == 2 && nch == 8) ec = launch_coop<2, 8>(ctx, c, Pc, dense, stream);
            else if (es == 2 && nch == 10) ec = launch_coop<2, 10>(ctx, c, Pc, dense, stream);
            else if (es == 2 && nch == 2) ec = launch_coop<2, 2>(ctx, c, Pc, dense, stream);
            else if (es == 4 && nch == 2) ec = launch_coop<4, 2>(ctx, c, Pc, dense, stream);
            else if (es == 4 && nch == 8) ec = launch_coop<4, 8>(ctx, c, Pc, dense, stream);
            if (ec == hipSuccess) {
                launch_finalize(es, p.partial, Pc, 1, d, (char *)y, reinterpret_cast<unsigned int *>(ctx->ws + COOP_EPOCH), stream);
                CLADA_CHECK_HIP(ctx, hipGetLastError());
                if (lists) {
                    hipLaunchKernelGGL(k_ffn_lists, dim3(1), dim3(1024), 0, stream, p.keep, B, F, active_idx, n_active, mask_bits);
                    CLADA_CHECK_HIP(ctx, hipGetLastError());
                }
                return CLADA_OK;
            }
            if (ec != hipErrorNotSupported) CLADA_CHECK_HIP(ctx, ec);
        }
    }
#define CLADA_DECODE_CASE(ES_, NCH_, NW_, GB_, UB_)                                        \
    if (es == ES_ && nch <= NCH_ && e == hipErrorInvalidValue)                             \
        e = launch_decode<ES_, NCH_, NW_, GB_, UB_>(p, P, B, dense, stream);
    if (es == 2 && nch == 8) {      // experimental launch shapes for the 4096-wide bf16 row
        switch (ctx->opt_decode_variant) {
        case 1: e = launch_decode<2, 8, 8, 1, 1>(p, P, B, dense, stream); break;
        case 2: e = launch_decode<2, 8, 8, 3, 1>(p, P, B, dense, stream); break;
        case 3: e = launch_decode<2, 8, 4, 4, 2>(p, P, B, dense, stream); break;
        case 4: e = launch_decode<2, 8, 4, 6, 3>(p, P, B, dense, stream); break;
        case 5: e = launch_decode<2, 8, 4, 3, 1>(p, P, B, dense, stream); break;
        case 6: e = launch_decode<2, 8, 4, 2, 1>(p, P, B, dense, stream); break;
        case 7: e = launch_decode<2, 8, 16, 1, 1>(p, P, B, dense, stream); break;
        default: break;
        }
    }
    CLADA_DECODE_CASE(2, 1, 8, 2, 2)
    CLADA_DECODE_CASE(2, 2, 8, 2, 2)
    CLADA_DECODE_CASE(2, 4, 8, 2, 2)
    CLADA_DECODE_CASE(2, 8, 8, 2, 1)
    CLADA_DECODE_CASE(2, 10, 8, 1, 1)
    CLADA_DECODE_CASE(2, 16, 8, 1, 1)
    CLADA_DECODE_CASE(4, 1, 8, 2, 2)
    CLADA_DECODE_CASE(4, 2, 8, 2, 2)
    CLADA_DECODE_CASE(4, 4, 8, 2, 2)
    CLADA_DECODE_CASE(4, 8, 8, 2, 1)
    CLADA_DECODE_CASE(4, 16, 8, 1, 1)
#undef CLADA_DECODE_CASE
    CLADA_CHECK_HIP(ctx, e);

    launch_finalize(es, p.partial, P, B, d, (char *)y, nullptr, stream);
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
