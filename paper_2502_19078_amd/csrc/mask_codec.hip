// Sparse (difference-coded) storage of activation masks.  The paper's limitations name the memory that
// stored masks take and its future work asks for a light-weight mask compression such as a sparse
// encoding; it defines no format.  The format here: the ascending positions at which a mask differs from
// a reference mask of the same layer (no reference = the all-zero mask), as gaps g_i = j_i - j_{i-1} - 1
// (j_{-1} = -1), each gap a little-endian base-128 number (7 value bits per byte, low group first, high
// bit set on every byte but the last).  A per-token mask costs d_ff/8 bytes as a bit mask whatever it
// holds (at the method's ~50 % sparsity that is within 1 % of the entropy bound, nothing beats it); coded
// against the layer's prefix-static mask or the previous token's mask it costs about one byte per neuron
// that changed.  One workgroup per mask, all integer and byte work, results exact.
#include "clada_internal.h"

namespace {

constexpr int NT = 1024;
constexpr int MAX_WORDS = CLADA_MAX_DFF / 32;

struct OpSum { __device__ static int id() { return 0; } __device__ static int f(int a, int b) { return a + b; } };
struct OpMax { __device__ static int id() { return -1; } __device__ static int f(int a, int b) { return a > b ? a : b; } };

// Exclusive scan of one int per thread over the workgroup under Op; *total gets the reduction of all.
template <typename Op>
__device__ __forceinline__ int block_excl_scan(int v, int *s_wave, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc = Op::f(inc, t);
    }
    int excl = __shfl_up(inc, 1);
    if (lane == 0) excl = Op::id();
    __syncthreads();                       // s_wave may still be read from a previous scan
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    int base = Op::id(), all = Op::id();
    for (int w = 0; w < NT / 64; ++w) {
        const int c = s_wave[w];
        if (w < wave) base = Op::f(base, c);
        all = Op::f(all, c);
    }
    *total = all;
    return Op::f(base, excl);
}

__device__ __forceinline__ int gap_bytes(int gap) { return 1 + (gap >= 128 ? 1 : 0) + (gap >= 16384 ? 1 : 0); }

// Thread t owns the words [t*per, (t+1)*per): the gap of its first position needs the last position of
// the threads before it (an exclusive max-scan), the byte offset an exclusive sum of the byte counts.
// One workgroup per mask: mask m at mask + m * words, its reference at ref + m * ref_stride (0: one for all),
// its stream at out + m * cap, its two counts at n_out + 2 m.
__global__ void __launch_bounds__(NT)
k_mask_sparse_encode(const unsigned int *__restrict__ mask, const unsigned int *__restrict__ ref, size_t ref_stride, int F,
                     unsigned char *__restrict__ out, int cap, int *__restrict__ n_out)
{
    __shared__ int s_wave[NT / 64];
    const int words = (F + 31) / 32;
    mask += (size_t)blockIdx.x * words;
    if (ref) ref += (size_t)blockIdx.x * ref_stride;
    out += (size_t)blockIdx.x * cap;
    n_out += 2 * (size_t)blockIdx.x;
    const int per = (words + NT - 1) / NT;
    const int w0 = min(words, (int)threadIdx.x * per), w1 = min(words, w0 + per);
    auto diff = [&](int w) {
        unsigned int v = mask[w] ^ (ref ? ref[w] : 0u);
        if (w == words - 1 && (F & 31)) v &= (1u << (F & 31)) - 1u;
        return v;
    };
    int last = -1;
    for (int w = w0; w < w1; ++w) {
        const unsigned int v = diff(w);
        if (v) last = 32 * w + 31 - __clz(v);
    }
    int dummy;
    const int prev0 = block_excl_scan<OpMax>(last, s_wave, &dummy);
    int bytes = 0, cnt = 0, prev = prev0;
    for (int w = w0; w < w1; ++w) {
        unsigned int v = diff(w);
        while (v) {
            const int pos = 32 * w + __ffs(v) - 1;
            bytes += gap_bytes(pos - prev - 1);
            prev = pos;
            ++cnt;
            v &= v - 1u;
        }
    }
    int total_bytes, total_cnt;
    int off = block_excl_scan<OpSum>(bytes, s_wave, &total_bytes);
    (void)block_excl_scan<OpSum>(cnt, s_wave, &total_cnt);
    if (total_bytes <= cap) {
        prev = prev0;
        for (int w = w0; w < w1; ++w) {
            unsigned int v = diff(w);
            while (v) {
                const int pos = 32 * w + __ffs(v) - 1;
                int gap = pos - prev - 1;
                while (gap >= 128) {
                    out[off++] = (unsigned char)((gap & 127) | 128);
                    gap >>= 7;
                }
                out[off++] = (unsigned char)gap;
                prev = pos;
                v &= v - 1u;
            }
        }
    }
    if (threadIdx.x == 0) {
        n_out[0] = total_bytes <= cap ? total_bytes : -1;
        n_out[1] = total_cnt;
    }
}

// Thread t owns the bytes [t*per, (t+1)*per) and decodes the numbers that END there (last byte = high bit
// clear; a number's earlier bytes may belong to the thread before).  The position of a number is one more
// than the sum of all gaps + 1 before it: an exclusive sum over the threads.  Sums saturate at F + 1, so a
// malformed stream can only name positions >= F, which are ignored; bytes after the last complete number
// are ignored as well.
__global__ void __launch_bounds__(NT)
k_mask_sparse_decode(const unsigned char *__restrict__ in, const int *__restrict__ n_bytes, size_t n_stride, int cap,
                     const unsigned int *ref, size_t ref_stride, int F, unsigned int *out)
{
    __shared__ int s_wave[NT / 64];
    __shared__ unsigned int s_bits[MAX_WORDS];
    const int words = (F + 31) / 32;
    in += (size_t)blockIdx.x * cap;
    n_bytes += (size_t)blockIdx.x * n_stride;
    if (ref) ref += (size_t)blockIdx.x * ref_stride;      // (out may be ref: every word is read before it is written)
    out += (size_t)blockIdx.x * words;
    for (int w = threadIdx.x; w < words; w += NT) s_bits[w] = 0u;
    const int n = min(max(n_bytes[0], 0), cap);
    const int per = (n + NT - 1) / NT;
    const int i0 = min(n, (int)threadIdx.x * per), i1 = min(n, i0 + per);
    auto number_ending_at = [&](int i) {      // at most three bytes (21 bits) per number
        int v = in[i];
        if (i >= 1 && (in[i - 1] & 128)) {
            v = (v << 7) | (in[i - 1] & 127);
            if (i >= 2 && (in[i - 2] & 128)) v = (v << 7) | (in[i - 2] & 127);
        }
        return v;
    };
    const int sat = F + 1;
    int adv = 0;
    for (int i = i0; i < i1; ++i)
        if (!(in[i] & 128)) adv = min(sat, adv + min(sat, number_ending_at(i) + 1));
    int total;
    int pos = block_excl_scan<OpSum>(adv, s_wave, &total) - 1;      // (also orders the zeroing of s_bits before the atomics)
    for (int i = i0; i < i1; ++i)
        if (!(in[i] & 128)) {
            pos = min(sat, pos + min(sat, number_ending_at(i) + 1));
            if (pos < F) atomicOr(&s_bits[pos >> 5], 1u << (pos & 31));
        }
    __syncthreads();
    for (int w = threadIdx.x; w < words; w += NT) {
        unsigned int v = (ref ? ref[w] : 0u) ^ s_bits[w];
        if (w == words - 1 && (F & 31)) v &= (1u << (F & 31)) - 1u;
        out[w] = v;
    }
}

}  // namespace

extern "C" size_t clada_mask_sparse_max_bytes(int32_t d_ff)
{
    if (d_ff < 1) return 0;
    // one byte per position, one more per gap >= 128, another per gap >= 16384 (such gaps use up that many positions)
    return (size_t)d_ff + (size_t)d_ff / 128 + (size_t)d_ff / 16384;
}

static clada_status check_codec(clada_ctx *ctx, int32_t d_ff, int32_t n_masks, int32_t stream_capacity, int64_t ref_stride)
{
    if (d_ff < 1 || d_ff > CLADA_MAX_DFF) return clada_fail(ctx, CLADA_ERR_SHAPE, "d_ff=%d outside [1,%d]", d_ff, CLADA_MAX_DFF);
    if (n_masks < 1 || n_masks > 65535) return clada_fail(ctx, CLADA_ERR_SHAPE, "n_masks=%d outside [1,65535]", n_masks);
    if (stream_capacity < 0) return clada_fail(ctx, CLADA_ERR_SHAPE, "stream_capacity=%d is negative", stream_capacity);
    if (ref_stride < 0) return clada_fail(ctx, CLADA_ERR_SHAPE, "ref_stride_words=%lld is negative", (long long)ref_stride);
    if (!ctx->ws) return clada_fail(ctx, CLADA_ERR_WORKSPACE, "the context has no workspace (no device)");
    return CLADA_OK;
}

extern "C" clada_status clada_mask_sparse_encode_batch(clada_ctx *ctx, const uint32_t *mask_bits, const uint32_t *ref_bits,
                                                       int64_t ref_stride_words, int32_t d_ff, int32_t n_masks,
                                                       uint8_t *stream, int32_t stream_capacity, int32_t *n_out,
                                                       void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    if (!mask_bits || !stream || !n_out) return clada_fail(ctx, CLADA_ERR_NULL, "mask_bits, stream or n_out is NULL");
    clada_status cs = check_codec(ctx, d_ff, n_masks, stream_capacity, ref_stride_words);
    if (cs != CLADA_OK) return cs;
    hipLaunchKernelGGL(k_mask_sparse_encode, dim3(n_masks), dim3(NT), 0, (hipStream_t)hip_stream, mask_bits, ref_bits,
                       (size_t)ref_stride_words, d_ff, stream, stream_capacity, n_out);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    return CLADA_OK;
}

extern "C" clada_status clada_mask_sparse_decode_batch(clada_ctx *ctx, const uint8_t *stream, const int32_t *n_bytes,
                                                       int64_t n_bytes_stride, int32_t stream_capacity,
                                                       const uint32_t *ref_bits, int64_t ref_stride_words, int32_t d_ff,
                                                       int32_t n_masks, uint32_t *mask_bits, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    if (!stream || !n_bytes || !mask_bits) return clada_fail(ctx, CLADA_ERR_NULL, "stream, n_bytes or mask_bits is NULL");
    clada_status cs = check_codec(ctx, d_ff, n_masks, stream_capacity, ref_stride_words);
    if (cs != CLADA_OK) return cs;
    if (n_bytes_stride < 1) return clada_fail(ctx, CLADA_ERR_SHAPE, "n_bytes_stride=%lld below 1", (long long)n_bytes_stride);
    hipLaunchKernelGGL(k_mask_sparse_decode, dim3(n_masks), dim3(NT), 0, (hipStream_t)hip_stream, stream, n_bytes,
                       (size_t)n_bytes_stride, stream_capacity, ref_bits, (size_t)ref_stride_words, d_ff, mask_bits);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    return CLADA_OK;
}

extern "C" clada_status clada_mask_sparse_encode(clada_ctx *ctx, const uint32_t *mask_bits, const uint32_t *ref_bits,
                                                 int32_t d_ff, uint8_t *stream, int32_t stream_capacity,
                                                 int32_t *n_out, void *hip_stream)
{
    return clada_mask_sparse_encode_batch(ctx, mask_bits, ref_bits, 0, d_ff, 1, stream, stream_capacity, n_out, hip_stream);
}

extern "C" clada_status clada_mask_sparse_decode(clada_ctx *ctx, const uint8_t *stream, const int32_t *n_bytes,
                                                 int32_t stream_capacity, const uint32_t *ref_bits, int32_t d_ff,
                                                 uint32_t *mask_bits, void *hip_stream)
{
    return clada_mask_sparse_decode_batch(ctx, stream, n_bytes, 1, stream_capacity, ref_bits, 0, d_ff, 1, mask_bits, hip_stream);
}
