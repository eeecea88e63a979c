// Prefill statistics (section 3.2.1, neuron-activation equation; algorithm
// "CLADA Inference", prefill phase): dense SwiGLU FFN over the prefix on the
// matrix cores with the per-neuron aggregates fused into the GEMM epilogue.
//
//   kernel 1 (gate+up): C_g = X W_gate^T and C_u = X W_up^T share the X tile;
//     both operands are K-contiguous (X [T][d], W [F][d]) so fragments come
//     straight from LDS.  Epilogue on the accumulators: a = SiLU(C_g),
//     h = a*C_u, per-neuron partial sums over the tile's tokens (|a|, a^2, h^2,
//     max|a|), the |a| pool, and h stored in the layer dtype for kernel 2.
//   kernel 2 (down): Y = H W_down, W_down tile transposed on its way into LDS.
//   kernel 3: fixed-order reduction of the per-token-tile partials,
//     A_j = sqrt(sum_t h_tj^2) * ||W_down[j,:]||_2.
// Tiles are 128x128x32, four wavefronts of 64x64, MFMA 32x32x16 (bf16) or
// 32x32x2 (fp32), fp32 accumulation.  Block ids are remapped so that the eight
// XCDs each walk their own range of neuron tiles (the weight tile stays in that
// XCD's L2 while the token tiles stream past it).
#include <math.h>

#include <type_traits>

#include "clada_internal.h"

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

constexpr int BM = 128, BN = 128;
// k-tile depth: 64 for bf16 (half as many barriers per flop), 32 for fp32 (LDS budget)
template <int ES> constexpr int BKV = (ES == 2) ? 64 : 32;

template <int ES> struct Tile {
    static constexpr int ROW = BKV<ES> * ES + 16;       // padded LDS row stride, bytes
    static constexpr int CHUNKS = BKV<ES> * ES / 16;    // 16-byte chunks per tile row
    static constexpr int PER_THREAD = BM * CHUNKS / 256; // chunks each thread moves per tile
};

// One k-tile of MFMAs for a 64x64 wave tile.  sa / sb point at the wave's first
// row of the A / B tile in LDS.
template <int ES, int NB>
__device__ __forceinline__ void mma_tile(const char *sa, const char *const (&sb)[NB], f32x16 (&acc)[NB][2][2], int lane)
{
    constexpr int ROW = Tile<ES>::ROW;
    const int r = lane & 31, q = lane >> 5;
    if (ES == 2) {
#pragma unroll
        for (int ks = 0; ks < BKV<ES> / 16; ++ks) {
            bf16x8 a[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
                a[mb] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(sa + (mb * 32 + r) * ROW + (ks * 16 + q * 8) * 2));
#pragma unroll
            for (int w = 0; w < NB; ++w)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) {
                    const bf16x8 bv = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(sb[w] + (nb * 32 + r) * ROW + (ks * 16 + q * 8) * 2));
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
                        acc[w][mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb], bv, acc[w][mb][nb], 0, 0, 0);
                }
        }
    } else {
#pragma unroll
        for (int ks = 0; ks < BKV<ES> / 2; ++ks) {
            float a[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
                a[mb] = *reinterpret_cast<const float *>(sa + (mb * 32 + r) * ROW + (ks * 2 + q) * 4);
#pragma unroll
            for (int w = 0; w < NB; ++w)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) {
                    const float bv = *reinterpret_cast<const float *>(sb[w] + (nb * 32 + r) * ROW + (ks * 2 + q) * 4);
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
                        acc[w][mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mb], bv, acc[w][mb][nb], 0, 0, 0);
                }
        }
    }
}

// SiLU of the prefill epilogues: hardware exp2 and reciprocal (a few ulp), a third of the instructions
// of the division form; +-inf and NaN behave as in g / (1 + exp(-g)).
__device__ __forceinline__ float silu_prefill(float g)
{
    return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * g));
}

// Tanh-form GELU the same way: g * sigmoid(2 sqrt(2/pi) (g + 0.044715 g^3)).
__device__ __forceinline__ float gelu_prefill(float g)
{
    const float u2 = 1.5957691216057308f * fmaf(0.044715f * g, g * g, g);
    return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * u2));
}

// Row of accumulator register r of a 32x32 MFMA block held by `lane`.
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// XCD-aware remap: consecutive block ids alternate over the 8 XCDs; give each XCD a
// contiguous run of tiles, token tile fastest.
__device__ __forceinline__ int remap_block(int id, int total)
{
    const int per = (total + 7) / 8;
    return (id & 7) * per + (id >> 3);
}

struct GateUpParams {
    const char *x, *wg, *wu;
    int T, d, F, n_tm, n_tn;
    float *part;        // [n_tm][4][F]  partial aggregates (sum|a|, sum a^2, max|a|, sum h^2)
    float *pool;        // [T][F] or nullptr
    char *hbuf;         // [T][Fp] layer dtype (Fp = F rounded up to BK, zero past F) or nullptr
    int Fp;             // F rounded up to a multiple of 64
    const float *b_in;  // non-gated family: input bias [F] or nullptr
    int relu;           // non-gated family: a = max(0, C_g + b_in), h = a (wu then aliases wg and C_u is ignored)
    int gelu;           // gated family: sigma = tanh-form GELU instead of SiLU
};

// Epilogue of the gate/up GEMM on the accumulators (shared by the fp32 and bf16 kernels):
// a = SiLU(C_g), h = a*C_u, per-neuron partial sums over the tile's tokens, |a| pool, h store.
template <int ES>
__device__ __forceinline__ void gateup_epilogue(const f32x16 (&acc)[2][2][2], const GateUpParams &p, int tm, int tn,
                                                int wm, int wn, int lane, int tid, float (&s_stat)[2][4][BN])
{
    // ------------------------------------------------------------------ epilogue
    const int n = lane & 31;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int jl = wn * 64 + nb * 32 + n;          // neuron inside the tile
        const int j = tn * BN + jl;
        float s_abs = 0.f, s_sq = 0.f, mx = 0.f, s_h2 = 0.f;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int t = tm * BM + wm * 64 + mb * 32 + acc_row(r, lane);
                float a, h;
                if (p.relu) {
                    const float g = acc[0][mb][nb][r] + ((p.b_in && j < p.F) ? p.b_in[j] : 0.0f);
                    a = g > 0.0f ? g : (g != g ? g : 0.0f);
                    h = a;
                } else {
                    a = p.gelu ? gelu_prefill(acc[0][mb][nb][r]) : silu_prefill(acc[0][mb][nb][r]);
                    h = a * acc[1][mb][nb][r];
                }
                if (t < p.T && j < p.F) {
                    const float aa = fabsf(a);
                    s_abs += aa;
                    s_sq = fmaf(a, a, s_sq);
                    mx = (aa > mx || aa != aa) ? aa : mx;
                    s_h2 = fmaf(h, h, s_h2);
                    if (p.pool) p.pool[(size_t)t * p.F + j] = aa;
                }
                if (p.hbuf && t < p.T && j < p.Fp) {
                    const float hv = j < p.F ? h : 0.0f;
                    if (ES == 4) reinterpret_cast<float *>(p.hbuf)[(size_t)t * p.Fp + j] = hv;
                    else reinterpret_cast<unsigned short *>(p.hbuf)[(size_t)t * p.Fp + j] = (unsigned short)f32_to_bf16_bits(hv);
                }
            }
        // lanes l and l^32 hold the same neuron
        s_abs += __shfl_xor(s_abs, 32);
        s_sq += __shfl_xor(s_sq, 32);
        s_h2 += __shfl_xor(s_h2, 32);
        const float mo = __shfl_xor(mx, 32);
        mx = (mo > mx || mo != mo) ? mo : mx;
        if (lane < 32) {
            s_stat[wm][0][jl] = s_abs;
            s_stat[wm][1][jl] = s_sq;
            s_stat[wm][2][jl] = mx;
            s_stat[wm][3][jl] = s_h2;
        }
    }
    __syncthreads();
    if (tid < BN) {
        const int j = tn * BN + tid;
        if (j < p.F) {
            float *dst = p.part + (size_t)tm * 4 * p.F + j;
            dst[0] = s_stat[0][0][tid] + s_stat[1][0][tid];
            dst[(size_t)p.F] = s_stat[0][1][tid] + s_stat[1][1][tid];
            const float m0 = s_stat[0][2][tid], m1 = s_stat[1][2][tid];
            dst[2 * (size_t)p.F] = (m1 > m0 || m1 != m1) ? m1 : m0;
            dst[3 * (size_t)p.F] = s_stat[0][3][tid] + s_stat[1][3][tid];
        }
    }
}

template <int ES>
__global__ void __launch_bounds__(256)
k_prefix_gateup(const GateUpParams p)
{
    constexpr int ROW = Tile<ES>::ROW, CH = Tile<ES>::CHUNKS, PT = Tile<ES>::PER_THREAD;
    __shared__ __align__(16) char s_a[BM * ROW];
    __shared__ __align__(16) char s_g[BN * ROW];
    __shared__ __align__(16) char s_u[BN * ROW];
    __shared__ float s_stat[2][4][BN];

    const int total = p.n_tm * p.n_tn;
    const int tile = remap_block(blockIdx.x, total);
    if (tile >= total) return;
    const int tm = tile % p.n_tm, tn = tile / p.n_tm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const size_t rowbytes = (size_t)p.d * ES;

    f32x16 acc[2][2][2];
#pragma unroll
    for (int w = 0; w < 2; ++w)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[w][mb][nb][r] = 0.0f;

    u32x4 ra[PT], rg[PT], ru[PT];
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int i = 0; i < PT; ++i) {
            const int c = tid + i * 256, row = c / CH, ch = c % CH;
            const int kbyte = kt * BKV<ES> * ES + ch * 16;
            const bool kin = (size_t)kbyte < rowbytes;
            const int t = tm * BM + row, j = tn * BN + row;
            u32x4 z = {0u, 0u, 0u, 0u};
            ra[i] = (kin && t < p.T) ? *reinterpret_cast<const u32x4 *>(p.x + (size_t)t * rowbytes + kbyte) : z;
            rg[i] = (kin && j < p.F) ? *reinterpret_cast<const u32x4 *>(p.wg + (size_t)j * rowbytes + kbyte) : z;
            ru[i] = (kin && j < p.F) ? *reinterpret_cast<const u32x4 *>(p.wu + (size_t)j * rowbytes + kbyte) : z;
        }
    };
    const int nk = (p.d + BKV<ES> - 1) / BKV<ES>;
    load_tile(0);
    for (int kt = 0; kt < nk; ++kt) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PT; ++i) {
            const int c = tid + i * 256, row = c / CH, ch = c % CH;
            *reinterpret_cast<u32x4 *>(s_a + row * ROW + ch * 16) = ra[i];
            *reinterpret_cast<u32x4 *>(s_g + row * ROW + ch * 16) = rg[i];
            *reinterpret_cast<u32x4 *>(s_u + row * ROW + ch * 16) = ru[i];
        }
        __syncthreads();
        if (kt + 1 < nk) load_tile(kt + 1);
        const char *const sb[2] = {s_g + wn * 64 * ROW, s_u + wn * 64 * ROW};
        mma_tile<ES, 2>(s_a + wm * 64 * ROW, sb, acc, lane);
    }

    gateup_epilogue<ES>(acc, p, tm, tn, wm, wn, lane, tid, s_stat);
}

// bf16 gate/up GEMM with direct-to-LDS loads and a three-stage pipeline: global_load_lds_dwordx4
// writes a wave's 64 x 16 bytes straight into LDS (no staging registers), two k-tiles are in
// flight while the third is multiplied, one raw barrier per k-tile.  A tile row is 128 bytes (64
// bf16), so rows are stored XOR-swizzled (16-byte chunk c of row r sits at position
// c ^ ((r >> 1) & 7): 16 consecutive rows read the same chunk from 16 different bank groups),
// done on the global-address side because the LDS side of the transfer is fixed to base + lane*16.
// Each stage is its own __shared__ array so the compiler can tell the stages apart and does not
// wait for in-flight transfers into the other stages before reading this one.  Needs d % 64 == 0.
constexpr int GU_TILE = 128 * 128;     // bytes of one operand tile: 128 rows x 64 bf16

__device__ __forceinline__ void lds_dma16(const char *gsrc, char *ldst)
{
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)gsrc,
                                     (void __attribute__((address_space(3))) *)ldst, 16, 0, 0);
}

__global__ void __launch_bounds__(256)
k_prefix_gateup_bf16(const GateUpParams p)
{
    __shared__ __align__(16) char s_st0[3 * GU_TILE];
    __shared__ __align__(16) char s_st1[3 * GU_TILE];
    __shared__ __align__(16) char s_st2[3 * GU_TILE];
    __shared__ float s_stat[2][4][BN];

    // Tile order inside an XCD's run: with at least 8 token tiles, blocks of 8 token tiles x 4
    // neuron tiles, so the 32 workgroups that share an L2 at any time re-use each X slice four
    // times and each weight slice eight times (token tile fastest would re-use only the weights).
    int tm, tn;
    if (p.n_tm % 8 == 0) {
        const int tn_pad = (p.n_tn + 3) / 4 * 4;
        const int o = remap_block(blockIdx.x, p.n_tm * tn_pad);
        const int sb = o >> 5, w = o & 31, tmb = p.n_tm >> 3;
        tm = (sb % tmb) * 8 + (w & 7);
        tn = (sb / tmb) * 4 + (w >> 3);
        if (tn >= p.n_tn) return;
    } else {
        const int total = p.n_tm * p.n_tn;
        const int tile = remap_block(blockIdx.x, total);
        if (tile >= total) return;
        tm = tile % p.n_tm;
        tn = tile / p.n_tm;
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const size_t rowbytes = (size_t)p.d * 2;

    f32x16 acc[2][2][2];
#pragma unroll
    for (int w = 0; w < 2; ++w)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[w][mb][nb][r] = 0.0f;

    // a wave moves 8-row pieces (1 KiB) of each operand tile: lane = (row lr, LDS position lp)
    const int lr = lane >> 3, lp = lane & 7;
    const char *gx[4], *gg[4], *gu[4];
#pragma unroll
    for (int c4 = 0; c4 < 4; ++c4) {
        const int row = 8 * (wave + 4 * c4) + lr;           // rows past T / F repeat the last valid row;
        const int t = min(tm * BM + row, p.T - 1);          // their products land in discarded outputs
        const int j = min(tn * BN + row, p.F - 1);
        const int koff = (lp ^ (4 * (wave & 1) + (lr >> 1))) * 16;      // position lp holds chunk lp ^ ((row >> 1) & 7)
        gx[c4] = p.x + (size_t)t * rowbytes + koff;
        gg[c4] = p.wg + (size_t)j * rowbytes + koff;
        gu[c4] = p.wu + (size_t)j * rowbytes + koff;
    }
    // (Every tile walks k in the same order on purpose: workgroups in step share their X and weight
    // slices in L2.  Starting each tile at its own k, to spread the memory channels that rows a
    // power of two apart map to, was measured 12 % slower.)
    const int nk = p.d / 64;
    auto issue = [&](char *st, int kt) {
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) {
            char *dst = st + (wave + 4 * c4) * 1024;
            lds_dma16(gx[c4] + (size_t)kt * 128, dst);
            lds_dma16(gg[c4] + (size_t)kt * 128, dst + GU_TILE);
            lds_dma16(gu[c4] + (size_t)kt * 128, dst + 2 * GU_TILE);
        }
    };
    // Fragment reads are issued as inline assembly: for an LDS read the compiler cannot prove
    // distinct from an in-flight direct-to-LDS transfer it inserts vmcnt(0), which would serialise
    // the pipeline; the hand-placed vmcnt above already orders the transfers of the stage read here.
    const int r32 = lane & 31, q = lane >> 5, sw = (r32 >> 1) & 7;
    const unsigned int a_off = (unsigned int)((wm * 64 + r32) * 128);
    const unsigned int b_off = (unsigned int)(GU_TILE + (wn * 64 + r32) * 128);
    // The reads of k-step ks+1 are in flight while the MFMAs of k-step ks run: LDS returns data in
    // order, so waiting for lgkmcnt <= 6 means the older set of six has landed.
    auto compute = [&](const char *st) {
        const unsigned int base = (unsigned int)(size_t)(const __attribute__((address_space(3))) char *)st;
        u32x4 fr[2][6];
#define GU_READ6(S, KS)                                                                                   \
        {                                                                                                 \
            const unsigned int pos = (unsigned int)(((2 * (KS) + q) ^ sw) * 16);                          \
            const unsigned int pa = base + a_off + pos, pb = base + b_off + pos;                          \
            asm volatile("ds_read_b128 %0, %6\n\t"                                                        \
                         "ds_read_b128 %1, %6 offset:4096\n\t"                                            \
                         "ds_read_b128 %2, %7\n\t"                                                        \
                         "ds_read_b128 %3, %7 offset:4096\n\t"                                            \
                         "ds_read_b128 %4, %7 offset:16384\n\t"                                           \
                         "ds_read_b128 %5, %7 offset:20480"                                                \
                         : "=&v"(fr[S][0]), "=&v"(fr[S][1]), "=&v"(fr[S][2]), "=&v"(fr[S][3]),            \
                           "=&v"(fr[S][4]), "=&v"(fr[S][5])                                               \
                         : "v"(pa), "v"(pb));                                                             \
        }
#define GU_WAIT(S, CNT)                                                                                   \
        asm volatile("s_waitcnt lgkmcnt(" #CNT ")"                                                        \
                     : "+v"(fr[S][0]), "+v"(fr[S][1]), "+v"(fr[S][2]), "+v"(fr[S][3]), "+v"(fr[S][4]),    \
                       "+v"(fr[S][5]));
#define GU_MMA(S)                                                                                         \
        {                                                                                                 \
            const bf16x8 fa[2] = {__builtin_bit_cast(bf16x8, fr[S][0]), __builtin_bit_cast(bf16x8, fr[S][1])}; \
            const bf16x8 fb[2][2] = {{__builtin_bit_cast(bf16x8, fr[S][2]), __builtin_bit_cast(bf16x8, fr[S][3])}, \
                                     {__builtin_bit_cast(bf16x8, fr[S][4]), __builtin_bit_cast(bf16x8, fr[S][5])}}; \
            _Pragma("unroll") for (int w = 0; w < 2; ++w)                                                 \
            _Pragma("unroll") for (int nb = 0; nb < 2; ++nb)                                              \
            _Pragma("unroll") for (int mb = 0; mb < 2; ++mb)                                              \
                acc[w][mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mb], fb[w][nb], acc[w][mb][nb], 0, 0, 0); \
        }
        GU_READ6(0, 0)
        GU_READ6(1, 1)
        GU_WAIT(0, 6)
        GU_MMA(0)
        GU_READ6(0, 2)
        GU_WAIT(1, 6)
        GU_MMA(1)
        GU_READ6(1, 3)
        GU_WAIT(0, 6)
        GU_MMA(0)
        GU_WAIT(1, 0)
        GU_MMA(1)
#undef GU_READ6
#undef GU_WAIT
#undef GU_MMA
    };
    // wait until this wave's transfers of tile k have landed (the 12 of tile k+1 may stay in
    // flight), meet the other waves, refill the stage consumed one step ago, multiply
    auto step = [&](int k, const char *cur, char *nxt) {
        if (k + 1 < nk) __builtin_amdgcn_s_waitcnt(0x0F7C);     // vmcnt(12)
        else            __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0)
        __builtin_amdgcn_s_barrier();
        if (k + 2 < nk) issue(nxt, k + 2);
        compute(cur);
    };
    issue(s_st0, 0);
    if (nk > 1) issue(s_st1, 1);
    for (int kt = 0; kt < nk; kt += 3) {
        step(kt, s_st0, s_st2);
        if (kt + 1 < nk) step(kt + 1, s_st1, s_st0);
        if (kt + 2 < nk) step(kt + 2, s_st2, s_st1);
    }
    gateup_epilogue<2>(acc, p, tm, tn, wm, wn, lane, tid, s_stat);
}

// Epilogue of the 256-token kernel for one wave: 128 tokens (rows tm128*128 ..) x 64 neurons, gate
// accumulators acc[0], up accumulators acc[1].  FULL = the whole block lies inside [T] x [F], so no
// element needs a bounds check.  Writes the per-neuron partial sums of these 128 tokens.
// SINGLE (non-gated family): the tile is 256 neurons wide and both accumulator sets are pre-activations, acc[w]
// of the neurons tn*256 + w*128 + ...
template <bool FULL, bool SINGLE>
__device__ __forceinline__ void wide_epilogue(const f32x16 (&acc)[2][4][2], const GateUpParams &p, int tm128, int tn,
                                              int wn, int lane)
{
    const int n = lane & 31;
    const int t0 = tm128 * 128 + 4 * (lane >> 5);          // row of accumulator register 0 of block mb = 0
    const size_t F1 = (size_t)p.F, Fp1 = (size_t)p.Fp;
#pragma unroll
    for (int wnb = 0; wnb < (SINGLE ? 4 : 2); ++wnb) {
        const int w = wnb >> 1, nb = wnb & 1;
        const int j = tn * (SINGLE ? 2 * BN : BN) + w * BN + wn * 64 + nb * 32 + n;
        const bool jok = FULL || j < p.F;
        const float bj = (p.relu && p.b_in && jok) ? p.b_in[j] : 0.0f;
        float s_abs = 0.f, s_sq = 0.f, mx = 0.f, s_h2 = 0.f;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
            float aa[16], hh[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float a, h;
                if (SINGLE || p.relu) {
                    const float g = acc[SINGLE ? w : 0][mb][nb][r] + bj;
                    a = g > 0.0f ? g : (g != g ? g : 0.0f);
                    h = a;
                } else {
                    a = p.gelu ? gelu_prefill(acc[0][mb][nb][r]) : silu_prefill(acc[0][mb][nb][r]);
                    h = a * acc[1][mb][nb][r];
                }
                aa[r] = fabsf(a);
                hh[r] = h;
                const int t = t0 + mb * 32 + 8 * (r >> 2) + (r & 3);
                if (FULL || (t < p.T && jok)) {
                    s_abs += aa[r];
                    s_sq = fmaf(a, a, s_sq);
                    mx = (aa[r] > mx || aa[r] != aa[r]) ? aa[r] : mx;
                    s_h2 = fmaf(h, h, s_h2);
                }
            }
            if (p.pool) {
                float *dst = p.pool + (size_t)(t0 + mb * 32) * F1 + j;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r >> 2) + (r & 3);
                    if (FULL || (t0 + mb * 32 + row < p.T && jok)) dst[row * F1] = aa[r];
                }
            }
            if (p.hbuf) {
                unsigned short *dst = reinterpret_cast<unsigned short *>(p.hbuf) + (size_t)(t0 + mb * 32) * Fp1 + j;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r >> 2) + (r & 3);
                    if (FULL || (t0 + mb * 32 + row < p.T && j < p.Fp))
                        dst[row * Fp1] = (unsigned short)f32_to_bf16_bits(jok ? hh[r] : 0.0f);
                }
            }
        }
        // lanes l and l^32 hold the same neuron
        s_abs += __shfl_xor(s_abs, 32);
        s_sq += __shfl_xor(s_sq, 32);
        s_h2 += __shfl_xor(s_h2, 32);
        const float mo = __shfl_xor(mx, 32);
        mx = (mo > mx || mo != mo) ? mo : mx;
        if (lane < 32 && jok && tm128 < p.n_tm) {
            float *dst = p.part + (size_t)tm128 * 4 * F1 + j;
            dst[0] = s_abs;
            dst[F1] = s_sq;
            dst[2 * F1] = mx;
            dst[3 * F1] = s_h2;
        }
    }
}

// The same GEMM with a 256-token x 128-neuron workgroup tile: four waves of 128 x (64 gate + 64 up)
// outputs, all 256 accumulator registers of a lane in use.  The 128 x 128 kernel above moves
// 144 KiB through LDS (fragment reads plus the transfers' writes) per 1024 clocks of MFMA issue,
// more than LDS delivers; a wave tile twice as tall needs a third less of both per flop.  k-tiles
// are 32 deep (64-byte rows, chunk c of row r at position c ^ ((r >> 2) & 3)) so that four stages
// of 32 KiB fit: at the barrier that certifies k-tile k+1 (placed between the two k-steps of
// k-tile k, so the first fragment reads of k+1 run under the MFMAs of k) k-tile k+2 is in flight
// and k+3 is issued into the stage k-1 has left.  Per-neuron partial sums are written per 128-token
// half (one wave row each), i.e. in the layout of the 128-row kernel.
constexpr int GW_STAGE = 32 * 1024;    // X 256 x 64 B | gate 128 x 64 B | up 128 x 64 B
constexpr int GW_G = 16 * 1024, GW_U = 24 * 1024;

// SINGLE: the non-gated family has one input matrix, so the second operand is the next 128 rows of the same
// matrix and the workgroup tile is 256 tokens x 256 neurons of one GEMM (nothing is computed twice).
template <bool SINGLE>
__global__ void __launch_bounds__(256)
k_prefix_gateup_bf16_wide(const GateUpParams p)
{
    __shared__ __align__(16) char s_w[4 * GW_STAGE];

    constexpr int TN = SINGLE ? 2 * BN : BN;                // neurons per workgroup tile
    const int n_tn = SINGLE ? (p.F + TN - 1) / TN : p.n_tn;
    const int n_tmw = (p.T + 255) / 256;
    int tm, tn;
    if (n_tmw % 8 == 0) {                                   // 8 token tiles x 4 neuron tiles per XCD at a time
        const int tn_pad = (n_tn + 3) / 4 * 4;
        const int o = remap_block(blockIdx.x, n_tmw * tn_pad);
        const int sb = o >> 5, w = o & 31, tmb = n_tmw >> 3;
        tm = (sb % tmb) * 8 + (w & 7);
        tn = (sb / tmb) * 4 + (w >> 3);
        if (tn >= n_tn) return;
    } else {
        const int total = n_tmw * n_tn;
        const int tile = remap_block(blockIdx.x, total);
        if (tile >= total) return;
        tm = tile % n_tmw;
        tn = tile / n_tmw;
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const size_t rowbytes = (size_t)p.d * 2;

    f32x16 acc[2][4][2];
#pragma unroll
    for (int w = 0; w < 2; ++w)
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[w][mb][nb][r] = 0.0f;

    // a wave moves 16-row pieces (1 KiB): lane = (row lane >> 2, LDS position lane & 3)
    const int lr = lane >> 2;
    const int koff = ((lane & 3) ^ ((lane >> 4) & 3)) * 16;
    const char *gx[4], *gg[2], *gu[2];
#pragma unroll
    for (int c = 0; c < 4; ++c) {                           // rows past T / F repeat the last valid row;
        const int t = min(tm * 256 + 16 * (wave + 4 * c) + lr, p.T - 1);   // their products land in discarded outputs
        gx[c] = p.x + (size_t)t * rowbytes + koff;
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int j = min(tn * TN + 16 * (wave + 4 * c) + lr, p.F - 1);
        gg[c] = p.wg + (size_t)j * rowbytes + koff;
        if (SINGLE) gu[c] = p.wg + (size_t)min(j + BN, p.F - 1) * rowbytes + koff;
        else gu[c] = p.wu + (size_t)j * rowbytes + koff;
    }
    const int nk = p.d / 32;
    // transfer i (0..7) of this wave for k-tile kt: four X pieces, two gate, two up
    auto dma_one = [&](auto ic, char *st, int kt) {
        constexpr int i = decltype(ic)::value;
        if constexpr (i < 4) lds_dma16(gx[i] + (size_t)kt * 64, st + (wave + 4 * i) * 1024);
        else if constexpr (i < 6) lds_dma16(gg[i - 4] + (size_t)kt * 64, st + GW_G + (wave + 4 * (i - 4)) * 1024);
        else lds_dma16(gu[i - 6] + (size_t)kt * 64, st + GW_U + (wave + 4 * (i - 6)) * 1024);
    };
    auto issue = [&](char *st, int kt) {
        dma_one(std::integral_constant<int, 0>{}, st, kt); dma_one(std::integral_constant<int, 1>{}, st, kt);
        dma_one(std::integral_constant<int, 2>{}, st, kt); dma_one(std::integral_constant<int, 3>{}, st, kt);
        dma_one(std::integral_constant<int, 4>{}, st, kt); dma_one(std::integral_constant<int, 5>{}, st, kt);
        dma_one(std::integral_constant<int, 6>{}, st, kt); dma_one(std::integral_constant<int, 7>{}, st, kt);
    };
    const int r32 = lane & 31, q = lane >> 5, sw = (r32 >> 2) & 3;
    const unsigned int lds0 = (unsigned int)(size_t)(const __attribute__((address_space(3))) char *)s_w;
    const unsigned int a_off = lds0 + (unsigned int)((wm * 128 + r32) * 64);
    const unsigned int b_off = lds0 + (unsigned int)(GW_G + (wn * 64 + r32) * 64);
    u32x4 fr[2][8];         // two fragment sets: 0..3 = X rows mb*32.., 4,5 = gate nb, 6,7 = up nb
    // Fragment reads are inline assembly: for an LDS read the compiler cannot prove distinct from an
    // in-flight direct-to-LDS transfer it inserts vmcnt(0), which would serialise the pipeline; the
    // hand-placed vmcnt + barrier already order the transfers of the stage read here.
#define GW_RD(S, I, ADDR, OFF) asm volatile("ds_read_b128 %0, %1 offset:" #OFF : "=v"(fr[S][I]) : "v"(ADDR));
#define GW_WAIT(S)                                                                                        \
    asm volatile("s_waitcnt lgkmcnt(0)"                                                                   \
                 : "+v"(fr[S][0]), "+v"(fr[S][1]), "+v"(fr[S][2]), "+v"(fr[S][3]), "+v"(fr[S][4]),        \
                   "+v"(fr[S][5]), "+v"(fr[S][6]), "+v"(fr[S][7]));
    // MFMA I (0..15) of a k-step: B fragment I / 4 (gate 0, gate 1, up 0, up 1) against X row block I % 4
#define GW_MMA1(S, I)                                                                                     \
    {                                                                                                     \
        constexpr int bi = (I) >> 2, w = bi >> 1, nb = bi & 1, mb = (I) & 3;                              \
        acc[w][mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                         \
            __builtin_bit_cast(bf16x8, fr[S][mb]), __builtin_bit_cast(bf16x8, fr[S][4 + bi]), acc[w][mb][nb], 0, 0, 0); \
    }
#define GW_MMA8(S, I0)                                                                                    \
    GW_MMA1(S, I0) GW_MMA1(S, I0 + 1) GW_MMA1(S, I0 + 2) GW_MMA1(S, I0 + 3)                               \
    GW_MMA1(S, I0 + 4) GW_MMA1(S, I0 + 5) GW_MMA1(S, I0 + 6) GW_MMA1(S, I0 + 7)
    // all eight reads of k-step ks of the stage at byte offset so (no MFMAs in between)
    auto read_all = [&](auto sc, u32x4 (&fr)[2][8], unsigned int so, int ks) {
        constexpr int S = decltype(sc)::value;
        const unsigned int pos = (unsigned int)(((2 * ks + q) ^ sw) * 16);
        const unsigned int pa = a_off + so + pos, pb = b_off + so + pos;
        GW_RD(S, 0, pa, 0) GW_RD(S, 1, pa, 2048) GW_RD(S, 2, pa, 4096) GW_RD(S, 3, pa, 6144)
        GW_RD(S, 4, pb, 0) GW_RD(S, 5, pb, 2048) GW_RD(S, 6, pb, 8192) GW_RD(S, 7, pb, 10240)
    };
    // One k-tile.  All four waves run in step, so whatever they issue in a burst queues up behind the
    // same LDS and the same texture unit while the matrix cores wait: fragment reads and transfers are
    // dealt out one at a time between MFMAs (sched_barrier keeps the compiler from regrouping) -- the
    // reads in the first half of each k-step so that the last one has eight MFMAs to land, the
    // transfers one per MFMA slot over the whole workgroup (wave w takes slots 4i + w).
    //   first half : MFMAs of k-step 0 (set 0), reads of k-step 1 into set 1, second half of the
    //                transfers of k-tile k+3
    //   barrier    : k-tile k+1 has landed for every wave and k-tile k is no longer read
    //   second half: MFMAs of k-step 1 (set 1), reads of k-step 0 of k-tile k+1 into set 0, first half
    //                of the transfers of k-tile k+4 into the stage of k
    auto ktile = [&](auto dac, auto dbc, auto vmc, u32x4 (&fr)[2][8], f32x16 (&acc)[2][4][2], int k) {
        constexpr bool DA = decltype(dac)::value, DB = decltype(dbc)::value;
        constexpr int VM = decltype(vmc)::value;
        const unsigned int cur = (unsigned int)((k & 3) * GW_STAGE), nxt = (unsigned int)(((k + 1) & 3) * GW_STAGE);
        char *sta = s_w + ((k + 3) & 3) * GW_STAGE, *stb = s_w + (k & 3) * GW_STAGE;
#define GW_SB __builtin_amdgcn_sched_barrier(0);
#define GW_SLOT_A(SL)                                                                                     \
        if (DA && ((SL) & 3) == wave) dma_one(std::integral_constant<int, 4 + (SL) / 4>{}, sta, k + 3);   \
        GW_MMA1(0, SL) GW_SB
#define GW_SLOT_B(SL)                                                                                     \
        if (DB && ((SL) & 3) == wave) dma_one(std::integral_constant<int, (SL) / 4>{}, stb, k + 4);       \
        GW_MMA1(1, SL) GW_SB
        {
            const unsigned int pos = (unsigned int)(((2 + q) ^ sw) * 16);
            const unsigned int pa = a_off + cur + pos, pb = b_off + cur + pos;
            GW_WAIT(0)
            GW_RD(1, 0, pa, 0)      GW_SLOT_A(0)
            GW_RD(1, 1, pa, 2048)   GW_SLOT_A(1)
            GW_RD(1, 2, pa, 4096)   GW_SLOT_A(2)
            GW_RD(1, 3, pa, 6144)   GW_SLOT_A(3)
            GW_RD(1, 4, pb, 0)      GW_SLOT_A(4)
            GW_RD(1, 5, pb, 2048)   GW_SLOT_A(5)
            GW_RD(1, 6, pb, 8192)   GW_SLOT_A(6)
            GW_RD(1, 7, pb, 10240)  GW_SLOT_A(7)
            GW_SLOT_A(8) GW_SLOT_A(9) GW_SLOT_A(10) GW_SLOT_A(11)
            GW_SLOT_A(12) GW_SLOT_A(13) GW_SLOT_A(14) GW_SLOT_A(15)
            GW_WAIT(1)                                      // every read of k-tile k is complete before the barrier
        }
        if (VM == 16)     __builtin_amdgcn_s_waitcnt(0x4F70);   // vmcnt(16): k-tile k+1 landed, k+2 and k+3 may fly
        else if (VM == 8) __builtin_amdgcn_s_waitcnt(0x0F78);
        else              __builtin_amdgcn_s_waitcnt(0x0F70);
        __builtin_amdgcn_s_barrier();
        {
            const unsigned int pos = (unsigned int)((q ^ sw) * 16);
            const unsigned int pa = a_off + nxt + pos, pb = b_off + nxt + pos;
            GW_RD(0, 0, pa, 0)      GW_SLOT_B(0)
            GW_RD(0, 1, pa, 2048)   GW_SLOT_B(1)
            GW_RD(0, 2, pa, 4096)   GW_SLOT_B(2)
            GW_RD(0, 3, pa, 6144)   GW_SLOT_B(3)
            GW_RD(0, 4, pb, 0)      GW_SLOT_B(4)
            GW_RD(0, 5, pb, 2048)   GW_SLOT_B(5)
            GW_RD(0, 6, pb, 8192)   GW_SLOT_B(6)
            GW_RD(0, 7, pb, 10240)  GW_SLOT_B(7)
            GW_SLOT_B(8) GW_SLOT_B(9) GW_SLOT_B(10) GW_SLOT_B(11)
            GW_SLOT_B(12) GW_SLOT_B(13) GW_SLOT_B(14) GW_SLOT_B(15)
        }
#undef GW_SLOT_A
#undef GW_SLOT_B
#undef GW_SB
    };
    using T_ = std::true_type; using F_ = std::false_type;
    issue(s_w, 0);
    issue(s_w + GW_STAGE, 1);                               // d >= 64: at least two k-tiles
    if (nk > 2) issue(s_w + 2 * GW_STAGE, 2);
    if (nk > 3) {                                           // first half of k-tile 3; the loop sends the second
        dma_one(std::integral_constant<int, 0>{}, s_w + 3 * GW_STAGE, 3); dma_one(std::integral_constant<int, 1>{}, s_w + 3 * GW_STAGE, 3);
        dma_one(std::integral_constant<int, 2>{}, s_w + 3 * GW_STAGE, 3); dma_one(std::integral_constant<int, 3>{}, s_w + 3 * GW_STAGE, 3);
    }
    // k-tile 0 of this wave has landed: the transfers issued after it may stay in flight
    if (nk > 3)      __builtin_amdgcn_s_waitcnt(0x4F74);    // vmcnt(20)
    else if (nk > 2) __builtin_amdgcn_s_waitcnt(0x4F70);    // vmcnt(16)
    else             __builtin_amdgcn_s_waitcnt(0x0F78);    // vmcnt(8)
    __builtin_amdgcn_s_barrier();
    read_all(std::integral_constant<int, 0>{}, fr, 0u, 0);
    using V16 = std::integral_constant<int, 16>; using V8 = std::integral_constant<int, 8>; using V0 = std::integral_constant<int, 0>;
    for (int k = 0; k + 4 < nk; ++k) ktile(T_{}, T_{}, V16{}, fr, acc, k);
    if (nk >= 4) ktile(T_{}, F_{}, V16{}, fr, acc, nk - 4);
    if (nk >= 3) ktile(F_{}, F_{}, V8{}, fr, acc, nk - 3);
    ktile(F_{}, F_{}, V0{}, fr, acc, nk - 2);
    {   // last k-tile: nothing left to fetch
        const unsigned int so = (unsigned int)(((nk - 1) & 3) * GW_STAGE);
        read_all(std::integral_constant<int, 1>{}, fr, so, 1);
        GW_WAIT(0)
        GW_MMA8(0, 0) GW_MMA8(0, 8)
        GW_WAIT(1)
        GW_MMA8(1, 0) GW_MMA8(1, 8)
    }
#undef GW_RD
#undef GW_WAIT
#undef GW_MMA1
#undef GW_MMA8

    // ------------------------------------------------------------------ epilogue: this wave's 128 tokens x 64 neurons
    const int tm128 = 2 * tm + wm;
    if (tm128 * 128 + 128 <= p.T && tn * TN + TN <= p.F) wide_epilogue<true, SINGLE>(acc, p, tm128, tn, wn, lane);
    else wide_epilogue<false, SINGLE>(acc, p, tm128, tn, wn, lane);
}

struct DownParams {
    const char *h, *wd;
    char *y;                       // [T][d] layer dtype, or nullptr
    const float *bias;             // output bias [d] of the non-gated family, or nullptr
    float *rowsq;                  // [n_tn][T] per column-tile sums of squares of the fp32 rows, or nullptr
    int T, d, F, Fp, n_tm, n_tn;   // Fp = F rounded up to a multiple of BK (row stride of h)
    float *part_out;               // split-K (256 x 256 kernel): fp32 partial outputs [S][T][d] instead of y / rowsq
    int S;                         // number of k ranges the neurons are split into (1 = no split)
};

// Row sums of squares of a 128 x 128 output tile held in the accumulators of four waves (2 x 2
// blocks of 32 x 32 each): 32-lane butterfly per row, then the two column halves in fixed order.
__device__ __forceinline__ void down_rowsq(const f32x16 (&acc)[2][2], const DownParams &p, int tm, int tn, int wm,
                                           int wn, int lane, int tid, float (&s_rs)[2][BM])
{
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float v = fmaf(acc[mb][0][r], acc[mb][0][r], acc[mb][1][r] * acc[mb][1][r]);
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 8);
            v += __shfl_xor(v, 4);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 1);
            if ((lane & 31) == 0) s_rs[wn][wm * 64 + mb * 32 + acc_row(r, lane)] = v;
        }
    __syncthreads();
    if (tid < BM) {
        const int t = tm * BM + tid;
        if (t < p.T) p.rowsq[(size_t)tn * p.T + t] = s_rs[0][tid] + s_rs[1][tid];
    }
}

template <int ES>
__global__ void __launch_bounds__(256)
k_prefix_down(const DownParams p)
{
    constexpr int ROW = Tile<ES>::ROW, CH = Tile<ES>::CHUNKS, PT = Tile<ES>::PER_THREAD;
    constexpr int VEC = 16 / ES;
    __shared__ __align__(16) char s_a[BM * ROW];
    __shared__ __align__(16) char s_b[BN * ROW];      // [n][k]: W_down tile transposed
    __shared__ float s_rs[2][BM];

    const int total = p.n_tm * p.n_tn;
    const int tile = remap_block(blockIdx.x, total);
    if (tile >= total) return;
    const int tm = tile % p.n_tm, tn = tile / p.n_tm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const size_t hrow = (size_t)p.Fp * ES, wrow = (size_t)p.d * ES;

    f32x16 acc[1][2][2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[0][mb][nb][r] = 0.0f;

    // B tile in global memory: BK rows (neurons) x BN columns -> BK * BN*ES/16 chunks
    constexpr int BCH = BN * ES / 16;                  // chunks per neuron row of the tile
    constexpr int BPT = BKV<ES> * BCH / 256;
    u32x4 ra[PT], rb[BPT];
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int i = 0; i < PT; ++i) {
            const int c = tid + i * 256, row = c / CH, ch = c % CH;
            const size_t kbyte = (size_t)kt * BKV<ES> * ES + ch * 16;
            const int t = tm * BM + row;
            u32x4 z = {0u, 0u, 0u, 0u};
            // rows of h are padded to a multiple of BK elements, zero-filled past F
            ra[i] = (t < p.T && kbyte < hrow) ? *reinterpret_cast<const u32x4 *>(p.h + (size_t)t * hrow + kbyte) : z;
        }
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            const int c = tid + i * 256, k = c / BCH, ch = c % BCH;
            const int j = kt * BKV<ES> + k;
            const size_t nbyte = (size_t)tn * BN * ES + ch * 16;
            u32x4 z = {0u, 0u, 0u, 0u};
            rb[i] = (j < p.F && nbyte < wrow) ? *reinterpret_cast<const u32x4 *>(p.wd + (size_t)j * wrow + nbyte) : z;
        }
    };
    const int nk = (p.F + BKV<ES> - 1) / BKV<ES>;
    load_tile(0);
    for (int kt = 0; kt < nk; ++kt) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PT; ++i) {
            const int c = tid + i * 256, row = c / CH, ch = c % CH;
            *reinterpret_cast<u32x4 *>(s_a + row * ROW + ch * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            const int c = tid + i * 256, k = c / BCH, ch = c % BCH;
            const unsigned int w[4] = {rb[i].x, rb[i].y, rb[i].z, rb[i].w};
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const int nloc = ch * VEC + e;
                if (ES == 4) *reinterpret_cast<unsigned int *>(s_b + nloc * ROW + k * 4) = w[e];
                else *reinterpret_cast<unsigned short *>(s_b + nloc * ROW + k * 2) = (unsigned short)(w[e >> 1] >> (16 * (e & 1)));
            }
        }
        __syncthreads();
        if (kt + 1 < nk) load_tile(kt + 1);
        const char *const sb[1] = {s_b + wn * 64 * ROW};
        mma_tile<ES, 1>(s_a + wm * 64 * ROW, sb, acc, lane);
    }
    if (p.rowsq) down_rowsq(acc[0], p, tm, tn, wm, wn, lane, tid, s_rs);
    if (!p.y) return;
    const int n = lane & 31;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int col = tn * BN + wn * 64 + nb * 32 + n;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int t = tm * BM + wm * 64 + mb * 32 + acc_row(r, lane);
                if (t < p.T && col < p.d) {
                    const float v = acc[0][mb][nb][r] + (p.bias ? p.bias[col] : 0.0f);
                    if (ES == 4) reinterpret_cast<float *>(p.y)[(size_t)t * p.d + col] = v;
                    else reinterpret_cast<unsigned short *>(p.y)[(size_t)t * p.d + col] = (unsigned short)f32_to_bf16_bits(v);
                }
            }
    }
}

// bf16 down projection Y = H W_down with a 64-deep k-tile: the W_down tile stays row-major
// ([k][n], as it lies in memory) in LDS and the K-major MFMA B-fragments come from
// ds_read_b64_tr_b16 transpose reads (in each 16-lane group lane t = 4r + c4 supplies row
// k0 + r, columns 4*c4..4*c4+3 and receives column t of rows k0..k0+3).
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
constexpr int DBK = 64;
constexpr int DA_PITCH = DBK * 2 + 16;          // h tile row pitch (bytes)
constexpr int DB_PITCH = BN * 2 + 32;           // W_down tile row pitch: 4 rows of a transpose read hit distinct banks

__global__ void __launch_bounds__(256)
k_prefix_down_bf16(const DownParams p)
{
    __shared__ __align__(16) char s_a[BM * DA_PITCH];
    __shared__ __align__(16) char s_b[DBK * DB_PITCH];
    __shared__ float s_rs[2][BM];

    const int total = p.n_tm * p.n_tn;
    const int tile = remap_block(blockIdx.x, total);
    if (tile >= total) return;
    const int tm = tile % p.n_tm, tn = tile / p.n_tm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const size_t hrow = (size_t)p.Fp * 2, wrow = (size_t)p.d * 2;

    f32x16 acc[2][2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.0f;

    u32x4 ra[4], rb[4];
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * 256;
            u32x4 z = {0u, 0u, 0u, 0u};
            {   // h tile: 128 rows x 8 chunks
                const int row = c >> 3, ch = c & 7;
                const size_t kbyte = (size_t)kt * DBK * 2 + ch * 16;
                const int t = tm * BM + row;
                ra[i] = (t < p.T && kbyte < hrow) ? *reinterpret_cast<const u32x4 *>(p.h + (size_t)t * hrow + kbyte) : z;
            }
            {   // W_down tile: 64 rows x 16 chunks
                const int k = c >> 4, ch = c & 15;
                const int j = kt * DBK + k;
                const size_t nbyte = (size_t)tn * BN * 2 + ch * 16;
                rb[i] = (j < p.F && nbyte < wrow) ? *reinterpret_cast<const u32x4 *>(p.wd + (size_t)j * wrow + nbyte) : z;
            }
        }
    };
    const int nk = (p.F + DBK - 1) / DBK;
    const int r32 = lane & 31, q = lane >> 5;
    const int g = lane >> 4, t16 = lane & 15;
    load_tile(0);
    for (int kt = 0; kt < nk; ++kt) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * 256;
            *reinterpret_cast<u32x4 *>(s_a + (c >> 3) * DA_PITCH + (c & 7) * 16) = ra[i];
            *reinterpret_cast<u32x4 *>(s_b + (c >> 4) * DB_PITCH + (c & 15) * 16) = rb[i];
        }
        __syncthreads();
        if (kt + 1 < nk) load_tile(kt + 1);
#pragma unroll
        for (int ks = 0; ks < DBK / 16; ++ks) {
            bf16x8 a[2], b[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
                a[mb] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(
                            s_a + (wm * 64 + mb * 32 + r32) * DA_PITCH + (ks * 16 + q * 8) * 2));
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const char *src = s_b + (ks * 16 + 8 * (g >> 1) + (t16 >> 2)) * DB_PITCH +
                                  (wn * 64 + nb * 32 + 16 * (g & 1) + 4 * (t16 & 3)) * 2;
                const s16x4_t b0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3))) *)src);
                const s16x4_t b1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3))) *)(src + 4 * DB_PITCH));
                const uint2 u0 = __builtin_bit_cast(uint2, b0), u1 = __builtin_bit_cast(uint2, b1);
                b[nb] = __builtin_bit_cast(bf16x8, u32x4{u0.x, u0.y, u1.x, u1.y});
            }
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb], b[nb], acc[mb][nb], 0, 0, 0);
        }
    }
    if (p.rowsq) down_rowsq(acc, p, tm, tn, wm, wn, lane, tid, s_rs);
    if (!p.y) return;
    const int n = lane & 31;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int col = tn * BN + wn * 64 + nb * 32 + n;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int t = tm * BM + wm * 64 + mb * 32 + acc_row(r, lane);
                if (t < p.T && col < p.d)
                    reinterpret_cast<unsigned short *>(p.y)[(size_t)t * p.d + col] =
                        (unsigned short)f32_to_bf16_bits(acc[mb][nb][r] + (p.bias ? p.bias[col] : 0.0f));
            }
    }
}

// bf16 down projection with a 256-token x 256-column workgroup tile (four waves of 128 x 128, all
// 256 accumulator registers of a lane), built like k_prefix_gateup_bf16_wide: four stages of 32-deep
// k-tiles filled by direct-to-LDS transfers, reads and transfers dealt out between MFMAs, one
// barrier per k-tile.  The h tile uses that kernel's layout.  The W_down tile stays row-major
// ([k][256 columns], 512 bytes a row); a transfer of 1 KiB carries two rows.  A transposing read
// takes, per pass, 64 bytes from each of four consecutive rows, so row k is placed such that its
// bank offset is 64 (k & 3): odd rows are stored rotated by 64 bytes inside their 512 (the
// rotation happens on the global-address side of the transfer), and every pair of rows is followed
// by 128 bytes of padding.  Needs d % 256 == 0 and d_ff % 32 == 0 (no k-tile reaches past d_ff).
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
constexpr int DW_PAIR = 1024 + 128;                 // two W_down rows + padding
constexpr int DW_B = 16 * 1024;                     // offset of the W_down tile in a stage
constexpr int DW_STAGE = DW_B + 16 * DW_PAIR;       // 34816 bytes

__global__ void __launch_bounds__(256)
k_prefix_down_bf16_wide(const DownParams p)
{
    __shared__ __align__(16) char s_w[4 * DW_STAGE];

    const int n_tmw = (p.T + 255) / 256, n_tnw = p.d / 256;
    int tm, tn, ks = 0;
    if (p.S > 1) {                                          // split-K: the S parts of a tile sit side by side
        const int total = n_tmw * n_tnw * p.S;
        const int o = remap_block(blockIdx.x, total);
        if (o >= total) return;
        ks = o % p.S;
        tm = (o / p.S) % n_tmw;
        tn = (o / p.S) / n_tmw;
    } else if (n_tmw % 8 == 0) {                            // 8 token tiles x 4 column tiles per XCD at a time
        const int tn_pad = (n_tnw + 3) / 4 * 4;
        const int o = remap_block(blockIdx.x, n_tmw * tn_pad);
        const int sb = o >> 5, w = o & 31, tmb = n_tmw >> 3;
        tm = (sb % tmb) * 8 + (w & 7);
        tn = (sb / tmb) * 4 + (w >> 3);
        if (tn >= n_tnw) return;
    } else {
        const int total = n_tmw * n_tnw;
        const int tile = remap_block(blockIdx.x, total);
        if (tile >= total) return;
        tm = tile % n_tmw;
        tn = tile / n_tmw;
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const size_t hrow = (size_t)p.Fp * 2, wrow = (size_t)p.d * 2;

    f32x16 acc[4][4];                                       // [token block mb][column block nb]
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.0f;

    // transfers of a wave per k-tile: four 16-row pieces of the h tile, four row pairs of W_down
    const char *gh[4], *gw[4];
    {
        const int lr = lane >> 2;
        const int koff = ((lane & 3) ^ ((lane >> 4) & 3)) * 16;
        const int half = lane >> 5, cidx = ((lane & 31) - 4 * half) & 31;     // LDS position p of an odd row holds chunk p - 4
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int t = min(tm * 256 + 16 * (wave + 4 * c) + lr, p.T - 1);  // rows past T repeat the last one: discarded outputs
            gh[c] = p.h + (size_t)t * hrow + koff;
            gw[c] = p.wd + (size_t)(2 * (wave + 4 * c) + half) * wrow + (size_t)tn * 512 + cidx * 16;
        }
    }
    // this workgroup's k-tiles [kt0, kt0 + nk) of the d_ff / 32 (d_ff % 32 == 0; the host keeps S <= d_ff / 32)
    const int nk_all = p.F / 32;
    const int kt0 = (int)((long long)ks * nk_all / p.S);
    const int nk = (int)((long long)(ks + 1) * nk_all / p.S) - kt0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        gh[c] += (size_t)kt0 * 64;
        gw[c] += (size_t)kt0 * 32 * wrow;
    }
    auto dma_one = [&](auto ic, char *st, int kt) {
        constexpr int i = decltype(ic)::value;
        if constexpr (i < 4) lds_dma16(gh[i] + (size_t)kt * 64, st + (wave + 4 * i) * 1024);
        else lds_dma16(gw[i - 4] + (size_t)kt * 32 * wrow, st + DW_B + (wave + 4 * (i - 4)) * DW_PAIR);
    };
    auto issue = [&](char *st, int kt) {
        dma_one(std::integral_constant<int, 0>{}, st, kt); dma_one(std::integral_constant<int, 1>{}, st, kt);
        dma_one(std::integral_constant<int, 2>{}, st, kt); dma_one(std::integral_constant<int, 3>{}, st, kt);
        dma_one(std::integral_constant<int, 4>{}, st, kt); dma_one(std::integral_constant<int, 5>{}, st, kt);
        dma_one(std::integral_constant<int, 6>{}, st, kt); dma_one(std::integral_constant<int, 7>{}, st, kt);
    };
    const unsigned int lds0 = (unsigned int)(size_t)(const __attribute__((address_space(3))) char *)s_w;
    // A fragments: as in the gate/up kernel
    const int r32 = lane & 31, q = lane >> 5, sw = (r32 >> 2) & 3;
    const unsigned int a_off = lds0 + (unsigned int)((wm * 128 + r32) * 64);
    // B fragments: in each 16-lane group lane t = 4r + c4 supplies row k0 + r, columns 4 c4 .. 4 c4 + 3,
    // and receives column t of rows k0 .. k0 + 3; group g covers columns 16 (g & 1) .., k half g >> 1
    const int t16 = lane & 15, g = lane >> 4, rr = t16 >> 2;
    const unsigned int b_lane = lds0 + (unsigned int)(DW_B + (4 * (g >> 1) + (rr >> 1)) * DW_PAIR + (rr & 1) * 512);
    unsigned int b_off[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
        b_off[nb] = b_lane + (unsigned int)((wn * 256 + nb * 64 + 32 * (g & 1) + 8 * (t16 & 3) + 64 * (rr & 1)) & 511);
    u32x4 fa[2][4];                                         // two fragment sets
    u32x2 fb[2][8];                                         // [set][2 nb + half]: rows k0..k0+3 and k0+4..k0+7
#define DW_WAIT(S)                                                                                        \
    asm volatile("s_waitcnt lgkmcnt(0)"                                                                   \
                 : "+v"(fa[S][0]), "+v"(fa[S][1]), "+v"(fa[S][2]), "+v"(fa[S][3]), "+v"(fb[S][0]),        \
                   "+v"(fb[S][1]), "+v"(fb[S][2]), "+v"(fb[S][3]), "+v"(fb[S][4]), "+v"(fb[S][5]),        \
                   "+v"(fb[S][6]), "+v"(fb[S][7]));
    // MFMA I (0..15) of a k-step: column block I / 4 against token block I % 4
#define DW_MMA1(S, I)                                                                                     \
    {                                                                                                     \
        constexpr int nb = (I) >> 2, mb = (I) & 3;                                                        \
        const u32x4 bv = {fb[S][2 * nb].x, fb[S][2 * nb].y, fb[S][2 * nb + 1].x, fb[S][2 * nb + 1].y};    \
        acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[S][mb]),      \
                                                              __builtin_bit_cast(bf16x8, bv), acc[mb][nb], 0, 0, 0); \
    }
    // read I (0..11) of k-step KS from the stage at byte offset so into set S: four A fragments, then the
    // eight halves of the B fragments (rows k0..k0+3 and k0+4..k0+7 of each 32-column block)
    auto rd_one = [&](auto sc, auto ic, auto ksc, u32x4 (&fa)[2][4], u32x2 (&fb)[2][8], unsigned int so) {
        constexpr int S = decltype(sc)::value, I = decltype(ic)::value, KS = decltype(ksc)::value;
        if constexpr (I < 4) {
            const unsigned int pa = a_off + so + (unsigned int)(((2 * KS + q) ^ sw) * 16);
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(fa[S][I]) : "v"(pa), "n"(I * 2048));
        } else {
            const unsigned int pb = b_off[(I - 4) >> 1] + so;
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(fb[S][I - 4]) : "v"(pb), "n"(KS * 9216 + (I & 1) * 2304));
        }
    };
    // the same for MFMA slot SL of a k-step: slots 12..15 carry no read
    auto rd_slot = [&](auto sc, auto slc, auto ksc, u32x4 (&fa)[2][4], u32x2 (&fb)[2][8], unsigned int so) {
        if constexpr (decltype(slc)::value < 12) rd_one(sc, slc, ksc, fa, fb, so);
    };
#define DW_RD(S, I, SO, KS) rd_slot(std::integral_constant<int, S>{}, std::integral_constant<int, I>{},   \
                                    std::integral_constant<int, KS>{}, fa, fb, SO);
#define DW_SB __builtin_amdgcn_sched_barrier(0);
    auto read_all = [&](auto sc, auto ksc, u32x4 (&fa)[2][4], u32x2 (&fb)[2][8], unsigned int so) {
        constexpr int S = decltype(sc)::value, KS = decltype(ksc)::value;
        DW_RD(S, 0, so, KS) DW_RD(S, 1, so, KS) DW_RD(S, 2, so, KS) DW_RD(S, 3, so, KS)
        DW_RD(S, 4, so, KS) DW_RD(S, 5, so, KS) DW_RD(S, 6, so, KS) DW_RD(S, 7, so, KS)
        DW_RD(S, 8, so, KS) DW_RD(S, 9, so, KS) DW_RD(S, 10, so, KS) DW_RD(S, 11, so, KS)
    };
    // one k-tile; the schedule is that of k_prefix_gateup_bf16_wide (twelve reads per k-step here)
    auto ktile = [&](auto dac, auto dbc, auto vmc, u32x4 (&fa)[2][4], u32x2 (&fb)[2][8], f32x16 (&acc)[4][4], int k) {
        constexpr bool DA = decltype(dac)::value, DB = decltype(dbc)::value;
        constexpr int VM = decltype(vmc)::value;
        const unsigned int cur = (unsigned int)((k & 3) * DW_STAGE), nxt = (unsigned int)(((k + 1) & 3) * DW_STAGE);
        char *sta = s_w + ((k + 3) & 3) * DW_STAGE, *stb = s_w + (k & 3) * DW_STAGE;
#define DW_SLOT_A(SL)                                                                                     \
        DW_RD(1, SL, cur, 1)                                                                              \
        if (DA && ((SL) & 3) == wave) dma_one(std::integral_constant<int, 4 + (SL) / 4>{}, sta, k + 3);   \
        DW_MMA1(0, SL) DW_SB
#define DW_SLOT_B(SL)                                                                                     \
        DW_RD(0, SL, nxt, 0)                                                                              \
        if (DB && ((SL) & 3) == wave) dma_one(std::integral_constant<int, (SL) / 4>{}, stb, k + 4);       \
        DW_MMA1(1, SL) DW_SB
        DW_WAIT(0)
        DW_SLOT_A(0) DW_SLOT_A(1) DW_SLOT_A(2) DW_SLOT_A(3) DW_SLOT_A(4) DW_SLOT_A(5) DW_SLOT_A(6) DW_SLOT_A(7)
        DW_SLOT_A(8) DW_SLOT_A(9) DW_SLOT_A(10) DW_SLOT_A(11) DW_SLOT_A(12) DW_SLOT_A(13) DW_SLOT_A(14) DW_SLOT_A(15)
        DW_WAIT(1)                                          // every read of k-tile k is complete before the barrier
        if (VM == 16)     __builtin_amdgcn_s_waitcnt(0x4F70);   // vmcnt(16): k-tile k+1 landed, k+2 and k+3 may fly
        else if (VM == 8) __builtin_amdgcn_s_waitcnt(0x0F78);
        else              __builtin_amdgcn_s_waitcnt(0x0F70);
        __builtin_amdgcn_s_barrier();
        DW_SLOT_B(0) DW_SLOT_B(1) DW_SLOT_B(2) DW_SLOT_B(3) DW_SLOT_B(4) DW_SLOT_B(5) DW_SLOT_B(6) DW_SLOT_B(7)
        DW_SLOT_B(8) DW_SLOT_B(9) DW_SLOT_B(10) DW_SLOT_B(11) DW_SLOT_B(12) DW_SLOT_B(13) DW_SLOT_B(14) DW_SLOT_B(15)
#undef DW_SLOT_A
#undef DW_SLOT_B
    };
    using T_ = std::true_type; using F_ = std::false_type;
    using V16 = std::integral_constant<int, 16>; using V8 = std::integral_constant<int, 8>; using V0 = std::integral_constant<int, 0>;
    issue(s_w, 0);
    if (nk > 1) issue(s_w + DW_STAGE, 1);
    if (nk > 2) issue(s_w + 2 * DW_STAGE, 2);
    if (nk > 3) {                                           // first half of k-tile 3; the loop sends the second
        dma_one(std::integral_constant<int, 0>{}, s_w + 3 * DW_STAGE, 3); dma_one(std::integral_constant<int, 1>{}, s_w + 3 * DW_STAGE, 3);
        dma_one(std::integral_constant<int, 2>{}, s_w + 3 * DW_STAGE, 3); dma_one(std::integral_constant<int, 3>{}, s_w + 3 * DW_STAGE, 3);
    }
    if (nk > 3)      __builtin_amdgcn_s_waitcnt(0x4F74);    // vmcnt(20): k-tile 0 of this wave has landed
    else if (nk > 2) __builtin_amdgcn_s_waitcnt(0x4F70);    // vmcnt(16)
    else if (nk > 1) __builtin_amdgcn_s_waitcnt(0x0F78);    // vmcnt(8)
    else             __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
    read_all(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, fa, fb, 0u);
    for (int k = 0; k + 4 < nk; ++k) ktile(T_{}, T_{}, V16{}, fa, fb, acc, k);
    if (nk >= 4) ktile(T_{}, F_{}, V16{}, fa, fb, acc, nk - 4);
    if (nk >= 3) ktile(F_{}, F_{}, V8{}, fa, fb, acc, nk - 3);
    if (nk >= 2) ktile(F_{}, F_{}, V0{}, fa, fb, acc, nk - 2);
    {   // last k-tile: nothing left to fetch
        const unsigned int so = (unsigned int)(((nk - 1) & 3) * DW_STAGE);
        read_all(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{}, fa, fb, so);
        DW_WAIT(0)
        DW_MMA1(0, 0) DW_MMA1(0, 1) DW_MMA1(0, 2) DW_MMA1(0, 3) DW_MMA1(0, 4) DW_MMA1(0, 5) DW_MMA1(0, 6) DW_MMA1(0, 7)
        DW_MMA1(0, 8) DW_MMA1(0, 9) DW_MMA1(0, 10) DW_MMA1(0, 11) DW_MMA1(0, 12) DW_MMA1(0, 13) DW_MMA1(0, 14) DW_MMA1(0, 15)
        DW_WAIT(1)
        DW_MMA1(1, 0) DW_MMA1(1, 1) DW_MMA1(1, 2) DW_MMA1(1, 3) DW_MMA1(1, 4) DW_MMA1(1, 5) DW_MMA1(1, 6) DW_MMA1(1, 7)
        DW_MMA1(1, 8) DW_MMA1(1, 9) DW_MMA1(1, 10) DW_MMA1(1, 11) DW_MMA1(1, 12) DW_MMA1(1, 13) DW_MMA1(1, 14) DW_MMA1(1, 15)
    }
#undef DW_WAIT
#undef DW_MMA1
#undef DW_RD
#undef DW_SB

    // ------------------------------------------------------------------ epilogue: 128 tokens x 128 columns of this wave
    const int n = lane & 31;
    const int t0 = tm * 256 + wm * 128 + 4 * (lane >> 5);
    const int c0 = tn * 256 + wn * 128;                     // one 128-column tile of the row-norm buffer
    if (p.part_out) {                                       // split-K: fp32 partial sums, reduced by k_prefix_down_combine
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            float *dst = p.part_out + ((size_t)ks * p.T + t0) * p.d + c0 + nb * 32 + n;
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = mb * 32 + 8 * (r >> 2) + (r & 3);
                    if (t0 + row < p.T) dst[(size_t)row * p.d] = acc[mb][nb][r];
                }
        }
        return;
    }
    if (p.rowsq) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float v = 0.0f;
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) v = fmaf(acc[mb][nb][r], acc[mb][nb][r], v);
                v += __shfl_xor(v, 16);
                v += __shfl_xor(v, 8);
                v += __shfl_xor(v, 4);
                v += __shfl_xor(v, 2);
                v += __shfl_xor(v, 1);
                const int t = t0 + mb * 32 + 8 * (r >> 2) + (r & 3);
                if (n == 0 && t < p.T) p.rowsq[(size_t)(c0 >> 7) * p.T + t] = v;
            }
    }
    if (!p.y) return;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
        const int col = c0 + nb * 32 + n;
        const float bv = p.bias ? p.bias[col] : 0.0f;
        unsigned short *dst = reinterpret_cast<unsigned short *>(p.y) + (size_t)t0 * p.d + col;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = mb * 32 + 8 * (r >> 2) + (r & 3);
                if (t0 + row < p.T) dst[(size_t)row * p.d] = (unsigned short)f32_to_bf16_bits(acc[mb][nb][r] + bv);
            }
    }
}

// Sum of the S split-K partial outputs [S][T][d] in ascending order, then what the direct epilogue does:
// y in bf16 (+ bias) and / or the per-row sums of squares of every 128-column tile.  A workgroup takes
// 8 rows x 128 columns: thread = (row tid >> 5, four columns 4 (tid & 31) ..).
__global__ void __launch_bounds__(256)
k_prefix_down_combine(const float *__restrict__ part, int S, int T, int d, char *__restrict__ y,
                      const float *__restrict__ bias, float *__restrict__ rowsq)
{
    const int t = blockIdx.x * 8 + (threadIdx.x >> 5);
    const int col = blockIdx.y * 128 + 4 * (threadIdx.x & 31);
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (t < T) {
        for (int k = 0; k < S; ++k) {
            const float4 v = *reinterpret_cast<const float4 *>(part + ((size_t)k * T + t) * d + col);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
    }
    if (rowsq) {
        float v = fmaf(s.x, s.x, fmaf(s.y, s.y, fmaf(s.z, s.z, s.w * s.w)));
        v += __shfl_xor(v, 16);
        v += __shfl_xor(v, 8);
        v += __shfl_xor(v, 4);
        v += __shfl_xor(v, 2);
        v += __shfl_xor(v, 1);
        if ((threadIdx.x & 31) == 0 && t < T) rowsq[(size_t)blockIdx.y * T + t] = v;
    }
    if (y && t < T) {
        if (bias) {
            const float4 b = *reinterpret_cast<const float4 *>(bias + col);
            s.x += b.x; s.y += b.y; s.z += b.z; s.w += b.w;
        }
        uint2 o;
        o.x = f32_to_bf16_bits(s.x) | (f32_to_bf16_bits(s.y) << 16);
        o.y = f32_to_bf16_bits(s.z) | (f32_to_bf16_bits(s.w) << 16);
        *reinterpret_cast<uint2 *>(y + ((size_t)t * d + col) * 2) = o;
    }
}

// One wave per neuron: ||W_down[j,:]||^2, then fold the token-tile partials (fixed order)
// and write the requested aggregates.
template <int ES>
__global__ void __launch_bounds__(256)
k_prefix_reduce(const char *__restrict__ wd, int d, int F, const float *__restrict__ part, int n_tm,
                const clada_prefix_out out)
{
    constexpr int VEC = 16 / ES;
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= F) return;
    float wn2 = 0.0f;
    if (out.A) {
        // the row in 16-byte chunks, lane l takes chunks l, l + 64, ...: eight loads in flight at a time
        const char *row = wd + (size_t)j * d * ES;
        const int nchunk = d * ES / 16;
        for (int c0 = lane; c0 < nchunk; c0 += 8 * 64) {
            u32x4 v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v[i] = c0 + 64 * i < nchunk ? *reinterpret_cast<const u32x4 *>(row + (size_t)(c0 + 64 * i) * 16)
                                            : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float w[VEC];
                unpack_row16(v[i], w);
#pragma unroll
                for (int e = 0; e < VEC; ++e) wn2 = fmaf(w[e], w[e], wn2);
            }
        }
        wn2 = wave_sum(wn2);
    }
    // token-tile partials: lane l takes tiles l, l + 64, ... (all loads of a wave in flight together),
    // then the lanes are folded in the fixed order of the wave reductions
    float s_abs = 0.f, s_sq = 0.f, mx = 0.f, s_h2 = 0.f;
    for (int tmi = lane; tmi < n_tm; tmi += 64) {
        const float *src = part + (size_t)tmi * 4 * F + j;
        s_abs += src[0];
        s_sq += src[(size_t)F];
        const float m = src[2 * (size_t)F];
        mx = (m > mx || m != m) ? m : mx;
        s_h2 += src[3 * (size_t)F];
    }
    s_abs = wave_sum(s_abs);
    s_sq = wave_sum(s_sq);
    s_h2 = wave_sum(s_h2);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const float m = __shfl_xor(mx, o);
        mx = (m > mx || m != m) ? m : mx;                 // a NaN sticks
    }
    if (lane == 0) {
        if (out.sum_abs_act) out.sum_abs_act[j] = s_abs;
        if (out.sum_sq_act) out.sum_sq_act[j] = s_sq;
        if (out.max_abs_act) out.max_abs_act[j] = mx;
        if (out.sum_sq_h) out.sum_sq_h[j] = s_h2;
        if (out.A) out.A[j] = sqrtf(s_h2) * sqrtf(wn2);
    }
}

}  // namespace

size_t clada_ws_prefix(int32_t d, int32_t d_ff, int32_t T, bool want_y)
{
    if (T <= 0) return 0;
    const size_t n_tm = (size_t)(T + BM - 1) / BM;
    size_t need = align_up(sizeof(float) * 4 * n_tm * d_ff, 256);
    if (want_y) need += align_up((size_t)T * align_up((size_t)d_ff, 64) * 4, 256) + clada_ws_down_splitk(d, d_ff, T);
    return need;
}

int clada_prefix_token_tiles(int T) { return (T + BM - 1) / BM; }

// Split-K factor of the 256 x 256 down projection for a shape that leaves compute units idle
// (fewer than 192 tiles): enough parts to reach about one workgroup per CU, every part at least
// eight 32-deep k-tiles, at most 8.  1 = no split (the shape does not qualify or does not need it).
int clada_prefix_down_splits(int d, int F, int T)
{
    if (T <= 0 || d % 256 != 0 || F % 32 != 0) return 1;
    const int tiles = ((T + 255) / 256) * (d / 256);
    if (tiles >= 192) return 1;
    int S = 256 / tiles;
    if (S > 8) S = 8;
    if (S > F / 256) S = F / 256;
    return S < 2 ? 1 : S;
}
size_t clada_ws_down_splitk(int d, int F, int T)
{
    const int S = clada_prefix_down_splits(d, F, T);
    return S > 1 ? align_up(sizeof(float) * (size_t)S * T * d, 256) : 0;
}
int clada_prefix_col_tiles(int d) { return (d + BN - 1) / BN; }

// Gate/up GEMM with the fused activation epilogue: part [n_tm][4][F] per-neuron partial
// aggregates (always written), pool [T][F] |a| or nullptr, hbuf [T][Fp] h in the layer dtype or
// nullptr (Fp = F rounded up to 64, zero past F).
hipError_t clada_prefix_gateup(const clada_layer *layer, const void *x, int T, float *part, float *pool,
                               char *hbuf, int tile_mode, hipStream_t stream)
{
    const int d = layer->d, F = layer->d_ff, es = (int)dtype_size(layer->dtype);
    GateUpParams g;
    const bool relu = layer->kind == CLADA_FFN_RELU;
    g.x = (const char *)x; g.wg = (const char *)layer->w_gate;
    g.wu = (const char *)(relu ? layer->w_gate : layer->w_up);
    g.relu = relu ? 1 : 0; g.b_in = relu ? layer->b_in : nullptr;
    g.gelu = layer->kind == CLADA_FFN_GEGLU ? 1 : 0;
    g.T = T; g.d = d; g.F = F; g.n_tm = (T + BM - 1) / BM; g.n_tn = (F + BN - 1) / BN;
    g.part = part; g.pool = pool; g.hbuf = hbuf;
    g.Fp = (int)align_up((size_t)F, 64);
    const int total = g.n_tm * g.n_tn;
    const int grid = (total + 7) / 8 * 8;
    const int total_blk = g.n_tm % 8 == 0 ? g.n_tm * ((g.n_tn + 3) / 4 * 4) : total;   // the bf16 kernel's padded tile order
    // tile_mode: 0 = choose, 1 = 128-token tiles, 2 = 256-token tiles (bf16, d % 64 == 0 only)
    const int n_tmw = (T + 255) / 256;
    const bool wide_ok = es == 2 && d % 64 == 0;
    const bool wide = wide_ok && (tile_mode == 2 || (tile_mode == 0 && T > 128));     // measured faster from T = 512 down
    if (wide && relu) {                                     // one GEMM over 256-neuron tiles
        const int n_tn2 = (F + 2 * BN - 1) / (2 * BN);
        const int blocks = n_tmw % 8 == 0 ? n_tmw * ((n_tn2 + 3) / 4 * 4) : n_tmw * n_tn2;
        hipLaunchKernelGGL(k_prefix_gateup_bf16_wide<true>, dim3((blocks + 7) / 8 * 8), dim3(256), 0, stream, g);
    }
    else if (wide) {
        const int blocks = n_tmw % 8 == 0 ? n_tmw * ((g.n_tn + 3) / 4 * 4) : n_tmw * g.n_tn;
        hipLaunchKernelGGL(k_prefix_gateup_bf16_wide<false>, dim3((blocks + 7) / 8 * 8), dim3(256), 0, stream, g);
    }
    else if (es == 4) hipLaunchKernelGGL(k_prefix_gateup<4>, dim3(grid), dim3(256), 0, stream, g);
    else if (d % 64 == 0) hipLaunchKernelGGL(k_prefix_gateup_bf16, dim3((total_blk + 7) / 8 * 8), dim3(256), 0, stream, g);
    else         hipLaunchKernelGGL(k_prefix_gateup<2>, dim3(grid), dim3(256), 0, stream, g);
    return hipGetLastError();
}

// Down projection of h [T][Fp]: y [T][d] in the layer dtype and/or rowsq [col tiles][T], the
// per-column-tile sums of squares of the fp32 output rows (either may be nullptr).
hipError_t clada_prefix_down(const clada_layer *layer, const char *h, int T, char *y, float *rowsq,
                             float *splitk_ws, int tile_mode, hipStream_t stream)
{
    const int d = layer->d, F = layer->d_ff, es = (int)dtype_size(layer->dtype);
    DownParams q;
    q.h = h; q.wd = (const char *)layer->w_down; q.y = y; q.rowsq = rowsq;
    q.bias = (layer->kind == CLADA_FFN_RELU && y) ? layer->b_out : nullptr;
    q.T = T; q.d = d; q.F = F; q.Fp = (int)align_up((size_t)F, 64);
    q.n_tm = (T + BM - 1) / BM; q.n_tn = (d + BN - 1) / BN;
    const int tot = q.n_tm * q.n_tn, grid = (tot + 7) / 8 * 8;
    // 256 x 256 tiles (bf16, d % 256 == 0, d_ff % 32 == 0): directly when they fill the chip, split along
    // d_ff into S parts with a combining pass when they would not (splitk_ws [S][T][d] fp32).
    // tile_mode 1 = 128 x 128 tiles always.
    const int n_tmw = (T + 255) / 256, n_tnw = d / 256;
    const bool wide_ok = es == 2 && d % 256 == 0 && F % 32 == 0 && tile_mode != 1;
    const int S = wide_ok && splitk_ws ? clada_prefix_down_splits(d, F, T) : 1;
    q.part_out = nullptr; q.S = 1;
    if (wide_ok && S > 1) {
        q.part_out = splitk_ws; q.S = S;
        hipLaunchKernelGGL(k_prefix_down_bf16_wide, dim3((n_tmw * n_tnw * S + 7) / 8 * 8), dim3(256), 0, stream, q);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k_prefix_down_combine, dim3((T + 7) / 8, d / 128), dim3(256), 0, stream, splitk_ws, S, T, d,
                           y, q.bias, rowsq);
    }
    else if (wide_ok && (tile_mode == 2 || n_tmw * n_tnw >= 192)) {
        const int blocks = n_tmw % 8 == 0 ? n_tmw * ((n_tnw + 3) / 4 * 4) : n_tmw * n_tnw;
        hipLaunchKernelGGL(k_prefix_down_bf16_wide, dim3((blocks + 7) / 8 * 8), dim3(256), 0, stream, q);
    }
    else if (es == 4) hipLaunchKernelGGL(k_prefix_down<4>, dim3(grid), dim3(256), 0, stream, q);
    else         hipLaunchKernelGGL(k_prefix_down_bf16, dim3(grid), dim3(256), 0, stream, q);
    return hipGetLastError();
}

extern "C" clada_status clada_prefix_stats(clada_ctx *ctx, const clada_layer *layer, const void *x,
                                           int32_t T, void *y, const clada_prefix_out *out,
                                           void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    clada_status st = clada_check_layer(ctx, layer);
    if (st != CLADA_OK) return st;
    if (!x || !out) return clada_fail(ctx, CLADA_ERR_NULL, "x or out is NULL");
    if (T < 1 || T > (1 << 20)) return clada_fail(ctx, CLADA_ERR_SHAPE, "T=%d outside [1,2^20]", T);
    if (!aligned16(x) || (y && !aligned16(y))) return clada_fail(ctx, CLADA_ERR_ALIGN, "x and y must be 16-byte aligned");
    const int d = layer->d, F = layer->d_ff;
    const size_t need = CLADA_WS_HEADER + clada_ws_prefix(d, F, T, y != nullptr);
    if (ctx->ws_bytes < need)
        return clada_fail(ctx, CLADA_ERR_WORKSPACE, "workspace %zu < %zu bytes needed", ctx->ws_bytes, need);
    const int es = (int)dtype_size(layer->dtype);
    const int n_tm = (T + BM - 1) / BM;
    char *ws = ctx->ws + CLADA_WS_HEADER;
    hipStream_t stream = (hipStream_t)hip_stream;

    float *part = reinterpret_cast<float *>(ws);
    char *hbuf = y ? ws + align_up(sizeof(float) * 4 * (size_t)n_tm * F, 256) : nullptr;
    CLADA_CHECK_HIP(ctx, clada_prefix_gateup(layer, x, T, part, out->abs_act_pool, hbuf, ctx->opt_prefix_tile, stream));
    if (y) {
        float *splitk = clada_ws_down_splitk(d, F, T)
                            ? reinterpret_cast<float *>(hbuf + align_up((size_t)T * align_up((size_t)F, 64) * 4, 256)) : nullptr;
        CLADA_CHECK_HIP(ctx, clada_prefix_down(layer, hbuf, T, (char *)y, nullptr, splitk, ctx->opt_prefix_tile, stream));
    }
    if (out->sum_abs_act || out->sum_sq_act || out->max_abs_act || out->sum_sq_h || out->A) {
        if (es == 4) hipLaunchKernelGGL(k_prefix_reduce<4>, dim3((F + 3) / 4), dim3(256), 0, stream,
                                        (const char *)layer->w_down, d, F, part, n_tm, *out);
        else         hipLaunchKernelGGL(k_prefix_reduce<2>, dim3((F + 3) / 4), dim3(256), 0, stream,
                                        (const char *)layer->w_down, d, F, part, n_tm, *out);
        CLADA_CHECK_HIP(ctx, hipGetLastError());
    }
    return CLADA_OK;
}
