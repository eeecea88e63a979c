// Internal declarations shared by the HIP sources of libclada (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "clada.h"

#define CLADA_OCC_SLOTS 32

struct clada_ctx {
    int device;
    int num_cu;
    size_t ws_bytes;
    char *ws;            // device workspace, 256-byte aligned; first CLADA_WS_HEADER bytes = counters
    int opt_decode_wgs_per_cu;   // launch shape of the decode kernel (clada_set_option)
    int opt_decode_b1;           // batch-1 split-d kernel: 0 off (generic kernels), 1 balancing where it pays, 2 never, 3 always
    int opt_decode_own_first;    // K0 of the balanced kernel; 0 = default
    int opt_decode_batched;      // 1: MFMA path for 2 <= B <= 16 (bf16), 0: generic kernels
    int opt_decode_stack;        // whole-stack calls: 0 = L per-layer calls, 1 = one persistent kernel, 2 = chained launches, 3 = lanes (default)
    int opt_decode_lane_occ2;    // lanes at B = 1, rows of 4, 5, 8 KiB: 1 = the instance of which two workgroups fit a compute unit
    int opt_decode_spin_limit;   // polls a balanced batch-1 kernel makes before it gives up (see clada.h)
    int opt_prefix_tile;         // gate/up prefill GEMM: 0 choose by T, 1 = 128-token tiles, 2 = 256-token tiles
    int opt_diag_events;         // 1: decode calls record HIP events around their kernels (clada_diag_kernel_times)
    hipEvent_t ev[4];            // start/stop of the main decode kernel, start/stop of the final reduction
    int capturing;               // a clada_graph_begin is open
    hipStream_t lane_stream[3];  // further lanes of the whole-stack calls (created at the first such call, default priority)
    hipEvent_t ev_lane[4];       // fork, and the join of every further lane
    // workgroups per compute unit of the balanced batch-1 kernel instances on this context's device
    // (asked of the runtime once per instance; the balanced kernel needs all its workgroups resident)
    const void *occ_fn[CLADA_OCC_SLOTS];
    int occ_val[CLADA_OCC_SLOTS];
    int n_occ;
    char err[512];
};

// Upper bound on the decode kernel's workgroup count (sizes the partial-y scratch).
#define CLADA_MAX_DECODE_WGS 512

// The first bytes of the workspace hold self-resetting arrival counters (zeroed
// once at clada_create); the scratch area proper starts after them.
#define CLADA_WS_HEADER (416 * 1024)
enum { CTR_SIGNALS = 0, CTR_DECODE = 64, CTR_PREFIX = 128, CTR_CALIB = 192 };  // int32 slots
// Control words of the cooperative decode kernels inside the header (byte offsets).
#define COOP_MAX_WGS 256
enum { COOP_EPOCH = 1024, COOP_FAULT = 1088, STACK_EPOCH = 1152,
       COOP_REC = 4096 /* 256 records of 8 bytes */, STACK_REC = 6144 /* 3 x 256 records */,
       STACK_KCNT = 12288 /* 3 x 256 int32 */,
       COOP_APUB = 16384 /* 256*64 tagged words of 8 bytes = 128 KiB */,
       STACK_APUB = 16384 + 131072 /* 2 x 128 KiB, ends at 400 KiB */ };

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

clada_status clada_fail(clada_ctx *ctx, clada_status s, const char *fmt, ...);

#define CLADA_CHECK_HIP(ctx, expr)                                                          \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess)                                                               \
            return clada_fail((ctx), CLADA_ERR_HIP, "%s failed: %s", #expr,                 \
                              hipGetErrorString(e_));                                       \
    } while (0)

static inline size_t dtype_size(int32_t t) { return t == CLADA_F32 ? 4 : 2; }
static inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// Validation shared by the FFN calls.
clada_status clada_check_layer(clada_ctx *ctx, const clada_layer *layer);
clada_status clada_require_swiglu(clada_ctx *ctx, const clada_layer *layer, const char *call);

// Batched (B >= 2, bf16) MFMA decode path; *ran tells whether the shape was eligible and it ran.
// list / list_n (device; nullptr for all neurons): run over the listed neurons only, all kept (dense must be set).
clada_status clada_decode_batched(clada_ctx *ctx, const clada_layer *layer, const void *x, int32_t B,
                                  const float *tau, void *y, unsigned char *keep, float *partial,
                                  char *scratch, bool dense, hipStream_t stream, bool *ran,
                                  const int32_t *list = nullptr, const int32_t *list_n = nullptr);
size_t clada_ws_decode_batched(int32_t d_ff);
size_t clada_ws_decode_batched_partial(int32_t d);
bool clada_decode_batched_eligible(const clada_ctx *ctx, const clada_layer *layer, int32_t B);
// Batch-1 decode over a neuron list with the streaming kernel, when the shape fits it (*ran).
hipError_t clada_decode_list_b1(clada_ctx *ctx, const clada_layer *layer, const void *x, const int32_t *idx,
                                const int32_t *n_active, float *partial, int *P_out, hipStream_t stream, bool *ran);
// Fixed-order sum of P partial y's [P][B][d] (fp32) into y (element size es).
void clada_launch_finalize(int es, const float *partial, int P, int B, int d, char *y, hipStream_t stream,
                           const float *bias = nullptr);

// Workspace needs of the individual calls (bytes beyond the header).
size_t clada_ws_decode(int32_t d, int32_t d_ff, int32_t B);
size_t clada_ws_signals(int32_t B, int32_t V);
size_t clada_ws_prefix(int32_t d, int32_t d_ff, int32_t T, bool want_y);
size_t clada_ws_calibrate(void);
size_t clada_ws_cett(int32_t d, int32_t d_ff, int32_t T);

// Prefill GEMMs shared by the prefix statistics and the CETT search (128 x 128 output tiles).
int clada_prefix_token_tiles(int T);
int clada_prefix_col_tiles(int d);
hipError_t clada_prefix_gateup(const clada_layer *layer, const void *x, int T, float *part, float *pool,
                               char *hbuf, int tile_mode, hipStream_t stream);
hipError_t clada_prefix_down(const clada_layer *layer, const char *h, int T, char *y, float *rowsq,
                             float *splitk_ws, int tile_mode, hipStream_t stream);
int clada_prefix_down_splits(int d, int F, int T);
size_t clada_ws_down_splitk(int d, int F, int T);

#ifdef __HIPCC__
// ---------------------------------------------------------------- device helpers
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// Eight bf16 values packed in 16 bytes -> fp32 (a bf16 is the top half of an fp32).
__device__ __forceinline__ void unpack_row16(const u32x4 v, float (&f)[8])
{
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}
// Four fp32 values in 16 bytes.
__device__ __forceinline__ void unpack_row16(const u32x4 v, float (&f)[4])
{
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
}

// 16-byte streaming load of weights that are read once (non-temporal: does not displace x and
// the partial sums in the caches).
__device__ __forceinline__ u32x4 ld_stream16(const char *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

// fp32 += bf16 pair . bf16 pair (exact products, fp32 accumulate).  The operands go through
// plain scalars: bit-casting a vector element expression directly was seen to pick lane 0.
__device__ __forceinline__ float dot2_bf16(unsigned int a, unsigned int b, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc, false);
}

template <int ES>
__device__ __forceinline__ float dot16(const u32x4 w, const u32x4 x, float acc)
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const unsigned int wk = w[k], xk = x[k];
        acc = ES == 2 ? dot2_bf16(wk, xk, acc) : fmaf(__uint_as_float(wk), __uint_as_float(xk), acc);
    }
    return acc;
}

// fp32 -> bf16 bits, round to nearest even (NaN stays NaN).
__device__ __forceinline__ unsigned int f32_to_bf16_bits(float f)
{
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Sum over the 64 lanes of a wavefront with DPP moves; every lane returns the
// total.  Fixed combination order, so the result is reproducible.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<0xB1, 0xf>(v);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E, 0xf>(v);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141, 0xf>(v);   // row_half_mirror
    v += dpp_move<0x140, 0xf>(v);   // row_mirror: every lane of a row holds the row's sum
    v += dpp_move<0x142, 0xa>(v);   // row_bcast15 into rows 1 and 3
    v += dpp_move<0x143, 0xc>(v);   // row_bcast31 into rows 2 and 3: lane 63 holds the total
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v)
{
    #pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// SiLU(g) = g * sigmoid(g), fp32.
__device__ __forceinline__ float silu_f32(float g) { return g / (1.0f + expf(-g)); }

// Tanh-form GELU, g/2 (1 + tanh(sqrt(2/pi) (g + 0.044715 g^3))), evaluated as g * sigmoid(2 u):
// 1 + tanh(u) = 2 sigmoid(2u), so no tanh is needed and the +-inf limits come out as for SiLU.
__device__ __forceinline__ float gelu_tanh_f32(float g)
{
    const float u2 = 1.5957691216057308f * fmaf(0.044715f * g, g * g, g);
    return g / (1.0f + expf(-u2));
}

// sigma of the gated families: SiLU (LLaMA / Mistral) or tanh-form GELU (Gemma)
__device__ __forceinline__ float gate_sigma_f32(float g, int gelu) { return gelu ? gelu_tanh_f32(g) : silu_f32(g); }
#endif
