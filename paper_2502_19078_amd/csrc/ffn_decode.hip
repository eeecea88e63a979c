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
    unsigned long long *rec;    // [P] keep mask of the workgroup's neurons (bit i = neuron blk + P*i)
    unsigned int *rec_tag;      // [P] epoch tag, stored (release) after the mask and activations
    float *apub;                // [P][64] published activations a_i of the workgroup's neurons
    float *partial;             // [P][d]
    unsigned int *done;         // [P] epoch tag once partial[p] is complete
    unsigned int *epoch;        // device-side call counter (survives graph replays)
    unsigned int *fin;          // arrival counter of finished workgroups
    unsigned char *keep;        // [F] or nullptr
    int d, F, K0, CW;           // CW = columns each workgroup reduces (multiple of 4)
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
    __shared__ float s_l2a[64];
    __shared__ int s_tmp[NW];
    __shared__ int s_misc[4];
    extern __shared__ __align__(16) unsigned char smem_coop[];
    float *s_red = reinterpret_cast<float *>(smem_coop);   // fold buffers, later the reduction staging

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int blk = blockIdx.x, P = gridDim.x;
    const int F = p.F;
    const int ni = blk < F ? (F - blk + P - 1) / P : 0;    // <= 56
    unsigned int ep = *p.epoch + 1u;                        // this call's tag (0 is never used)
    if (ep == 0u) ep = 1u;
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
    if (!DENSE && wave == 0) {                              // publish activations and mask, then the tag
        if (lane < ni) p.apub[blk * 64 + lane] = s_a[lane];
        if (lane == 0) {
            p.rec[blk] = mask;
            __hip_atomic_store(p.rec_tag + blk, ep, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    float acc[NCH][VEC];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[c][e] = 0.0f;

    auto updown = [&](int row_j, float a) {
        const size_t off = (size_t)row_j * ROWB + loff;
        u32x4 ub[NCH], db[NCH];
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
        updown(blk + P * i, s_a[i]);
    }

    // ------------------------------------------- share of the pooled surplus
    int n2 = 0;
    if (!DENSE) {
        unsigned long long mq = 0ull;
        if (tid < P) {
            const unsigned int *r = p.rec_tag + tid;
            while (__hip_atomic_load(r, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) != ep) __builtin_amdgcn_s_sleep(2);
            mq = __hip_atomic_load(p.rec + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        const int kq = __popcll(mq);
        const int oq = min(kq, p.K0), sq = kq - oq;
        int K, S, Etot;
        const int kpre = block_excl_scan(kq, tid, s_tmp, NW, &K);
        const int spre = block_excl_scan(sq, tid, s_tmp, NW, &S);
        // target count of workgroup q: floor((q+1)K/P) - floor(qK/P); extra beyond its own first rows
        const int tgt = tid < P ? (int)(((long long)(tid + 1) * K) / P - ((long long)tid * K) / P) : 0;
        const int eq = max(0, tgt - oq);
        const int epre = block_excl_scan(eq, tid, s_tmp, NW, &Etot);
        (void)kpre; (void)Etot;
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
            s_l2a[r - lo] = __hip_atomic_load(p.apub + tid * 64 + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        const int shift = own % NW;                         // wave that would take list entry `own`
        for (int r = (wave - shift + NW) % NW; r < n2; r += NW) updown(s_l2row[r], s_l2a[r]);
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
        if (lane == 0) __hip_atomic_store(p.done + blk, ep, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ------------------------------------ cross-workgroup reduction of this workgroup's columns
    // s_red is free again: [P][CW] staging, then a two-level fixed-order sum over q.
    const int CW = p.CW, c0 = blk * CW;
    if (tid < P) {
        const unsigned int *dn = p.done + tid;
        while (__hip_atomic_load(dn, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) != ep) __builtin_amdgcn_s_sleep(2);
        for (int c = 0; c < CW; c += 4) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c0 + c < p.d) {
                const float *src = p.partial + (size_t)tid * p.d + c0 + c;
                v.x = __hip_atomic_load(src + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                v.y = __hip_atomic_load(src + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                v.z = __hip_atomic_load(src + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                v.w = __hip_atomic_load(src + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            *reinterpret_cast<float4 *>(s_red + tid * CW + c) = v;
        }
    }
    __syncthreads();
    // level 1: thread (g, c) adds 16 consecutive q; level 2: thread c adds the 16 group sums
    const int ngrp = (P + 15) / 16;
    for (int idx = tid; idx < ngrp * CW; idx += NW * 64) {
        const int g = idx / CW, c = idx - g * CW;
        float sum = 0.0f;
        const int q1 = min(P, g * 16 + 16);
        for (int q = g * 16; q < q1; ++q) sum += s_red[q * CW + c];
        s_red[P * CW + idx] = sum;
    }
    __syncthreads();
    if (tid < CW && c0 + tid < p.d) {
        float sum = 0.0f;
        for (int g = 0; g < ngrp; ++g) sum += s_red[P * CW + g * CW + tid];
        if (ES == 4) reinterpret_cast<float *>(p.y)[c0 + tid] = sum;
        else reinterpret_cast<unsigned short *>(p.y)[c0 + tid] = (unsigned short)f32_to_bf16_bits(sum);
    }
    if (tid == 0) {
        const unsigned int prev = atomicAdd(p.fin, 1u);
        if (prev == (unsigned int)P - 1u) {                 // everyone has read the epoch long ago
            *p.fin = 0u;
            __hip_atomic_store(p.epoch, ep, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
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

// Cooperative launch; returns hipErrorNotSupported when the shape is not eligible.
template <int ES, int NCH>
hipError_t launch_coop(clada_ctx *ctx, const CoopParams &p, int P, bool dense, hipStream_t st)
{
    constexpr int NW = 8, VEC = 16 / ES;
    const size_t fold = sizeof(float) * (size_t)(NW / 2) * NCH * 64 * VEC;
    const size_t red = sizeof(float) * ((size_t)P * p.CW + (size_t)((P + 15) / 16) * p.CW);
    const size_t lds = fold > red ? fold : red;
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
        int Pc = ctx->num_cu < COOP_MAX_WGS ? ctx->num_cu : COOP_MAX_WGS;
        if (Pc > F) Pc = F;
        const int ni_c = (F + Pc - 1) / Pc;
        const int CW = ((d + Pc - 1) / Pc + 3) / 4 * 4;
        if (ni_c <= 56 && CW <= 32) {
            CoopParams c;
            c.wg = p.wg; c.wu = p.wu; c.wd = p.wd; c.x = p.x; c.tau = tau; c.y = (char *)y;
            c.rec = reinterpret_cast<unsigned long long *>(ctx->ws + COOP_REC);
            c.rec_tag = reinterpret_cast<unsigned int *>(ctx->ws + COOP_REC_TAG);
            c.apub = reinterpret_cast<float *>(ctx->ws + COOP_APUB);
            c.partial = p.partial;
            c.done = reinterpret_cast<unsigned int *>(ctx->ws + COOP_DONE);
            c.epoch = reinterpret_cast<unsigned int *>(ctx->ws + COOP_EPOCH);
            c.fin = reinterpret_cast<unsigned int *>(ctx->ws + COOP_FIN);
            c.keep = p.keep;
            c.d = d; c.F = F; c.CW = CW;
            c.K0 = ctx->opt_decode_own_first > 0 ? ctx->opt_decode_own_first : (ni_c / 6 > 1 ? ni_c / 6 : 1);
            hipError_t ec = hipErrorNotSupported;
            if (es == 2 && nch == 8) ec = launch_coop<2, 8>(ctx, c, Pc, dense, stream);
            else if (es == 2 && nch == 10) ec = launch_coop<2, 10>(ctx, c, Pc, dense, stream);
            else if (es == 2 && nch == 2) ec = launch_coop<2, 2>(ctx, c, Pc, dense, stream);
            else if (es == 4 && nch == 2) ec = launch_coop<4, 2>(ctx, c, Pc, dense, stream);
            else if (es == 4 && nch == 8) ec = launch_coop<4, 8>(ctx, c, Pc, dense, stream);
            if (ec == hipSuccess) {
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
