// Batched (2 <= B <= 16) thresholded sparse SwiGLU FFN at decode time on the matrix cores
// (algorithm "CLADA Inference", generation phase; bf16 layers).  With B tokens every weight
// element feeds B multiply-adds, which the vector ALUs cannot sustain at HBM speed, so the
// three projections run as MFMA 16x16x32 (bf16 in, fp32 accumulate) with the tokens as the
// 16-wide M dimension.  Weights are still read once, and only for neurons kept by at least
// one token (the union); every output row uses its own mask.  The GELU-gated family differs in
// sigma only; the non-gated ReLU family has no up projection: kernel A runs gate tiles alone and
// writes h = max(0, g + b_in) with the masks, and b_out is added by kernel C.
//
//   kernel A (gate + up -> h): workgroup p owns a contiguous run of neurons (dealt out evenly, to
//     within one), taken 16 at a time.  Its waves (8; 5 for 5 and 10 KiB rows) split the d (= K)
//     dimension: wave w keeps its slice of x as MFMA A-fragments in registers for the whole kernel
//     and streams its slice of the 16 weight rows as B-fragments (whole-KiB pieces of a row per
//     load instruction, turned into the operand layout through a wave-private LDS tile).  The
//     partial 16x16 tiles of the waves are summed through LDS in fixed order; sigma, the per-token
//     fp32 compare and the per-neuron 16-bit keep masks follow.  The neurons of gate tile i that at
//     least one token keeps (the union) are compacted by ballot and form up tile i: the same MFMA
//     loop over their W_up rows gives u, and h = keep ? a*u : 0 goes to a [d_ff][16] fp32 buffer
//     (the 16 tokens of a neuron = one 64-byte line).  Gate and up tiles alternate (G0 G1 U0 G2 U1
//     ...), so the stream of row loads does not drain between the two projections.  The workgroup
//     also leaves the list of its union-kept neurons, ascending, and their count for kernel B.
//   kernel B (down): 2-D split -- column groups of 256 x row groups (a fixed range of neuron
//     indices each: the lists of the gate/up workgroups that own them, laid end to end), so only
//     R partial y's exist instead of one per workgroup.  Work is dealt to the waves in units of 32
//     neurons x 128 columns (wave w: column half w & 1, neuron blocks w >> 1, + 4, ...).  W_down
//     rows arrive as 256-byte segments, are staged per wave in LDS and read
//     back K-major with ds_read_b64_tr_b16 as MFMA B-fragments; h is split into bf16 hi + lo
//     A-fragments (two MFMAs), so the down projection keeps ~fp32 accuracy of h.
//   kernel C: k_ffn_finalize adds the R partials in fixed order.
#include <atomic>

#include "clada_internal.h"

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;

struct BatParams {
    const char *wg, *wu, *wd, *x;
    const float *tau;           // [B]
    float *hbuf;                // [F][16] fp32 (neuron-major: one 64-byte line per neuron), written for union-kept neurons only
    int *ulist;                 // [F] union-kept neurons: gate/up workgroup q writes its own, ascending, from
                                //     the first neuron it owns (q * F / P) on
    int *ucnt;                  // [P] how many each wrote
    unsigned char *keep;        // [B][F] or nullptr
    float *partial;             // [RG][B][d]
    int d, F, B, P, RG, CG;
    int gelu;                   // sigma = tanh-form GELU instead of SiLU
    const float *b_in;          // non-gated family: input bias [F] or nullptr
    const int *list, *list_n;   // prefix-static run (with DENSE): the neurons are the list_n[0] entries of list
                                // (device), every one kept by every token; nullptr: all F neurons
};

__device__ __forceinline__ f32x4 mfma16(const u32x4 a, const u32x4 b, const f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// a line of zeros in global memory (never written): what a load of a row that does not exist reads
__device__ __align__(16) unsigned int k_zero16[4] = {0u, 0u, 0u, 0u};

// first neuron of gate/up workgroup w of P (w = P: d_ff)
__host__ __device__ __forceinline__ int bat_run_lo(int w, int F, int P) { return (int)((long long)w * F / P); }

constexpr int MAX_TILES = 4;    // 16-neuron tiles per workgroup in kernel A (one 64-lane ballot compacts them)

// NW waves split d; KSTEPS = k-steps of 32 per wave: d = NW * KSTEPS * 32.  (NW = 5 gives the 5 and
// 10 KiB rows whole-KiB slices; with 8 waves they would be 640 bytes, which streams slower.)
// LIST (with DENSE): the neurons are the entries of p.list, looked up through LDS; without it neuron
// indices are plain arithmetic on the run's start (fewer registers: the 10 and 16 KiB rows need that).
// RELU: the non-gated family (gate tiles only).  A template flag: as a run-time one it cost the
// 10 and 16 KiB rows ~25 registers and pushed them into scratch (52 -> 68 us at the 13B shape).
template <int KSTEPS, int NW, bool DENSE, bool LIST = false, bool RELU = false>
__global__ void __launch_bounds__(NW * 64)
k_bat_gateup(const BatParams p)
{
    static_assert(!LIST || DENSE, "a list run keeps every listed neuron");
    static_assert(NW >= 4 && NW <= 8, "the tile reductions run on waves 0..3");
    __shared__ float s_part[2][NW][256];
    __shared__ float s_a[MAX_TILES][16][16];
    __shared__ int s_km[MAX_TILES * 16];
    __shared__ int s_ul[MAX_TILES * 16];
    __shared__ int s_ku[MAX_TILES];
    __shared__ int s_nl[MAX_TILES * 16];                    // neuron index of every entry of the round

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, q = lane >> 4;
    const int blk = blockIdx.x, P = gridDim.x;
    const int d = p.d, F = p.F, B = p.B;
    const size_t rowb = (size_t)d * 2;
    // This wave's k-slice of every row is SLICE bytes, taken in NPART parts of PB <= 1024 bytes.  The
    // loads of eight rows' parts (8 PB bytes) are packed into NL = PB / 128 full instructions of
    // 64 x 16 bytes: lane l of instruction i takes byte 1024 i + 16 l of the eight parts laid end
    // to end, i.e. contiguous pieces of PB bytes (or the two ends of neighbouring rows) -- measured
    // 6.6 TB/s for whole-KiB pieces against 5.6 TB/s for 16 rows x 64 bytes per instruction, which
    // is what the MFMA operand layout would ask for.  The wave then turns 16 such rows into
    // B-fragments through its private LDS tile: row r is written contiguously at r * PITCH, and lane
    // (neuron n, k-group q) reads chunk q * SP + ks of row n for k-step ks.  The order of k within the
    // slice is free as long as x uses the same one.  PITCH = PB + 16 keeps both directions free of
    // bank conflicts.
    constexpr int SLICE = KSTEPS * 64;
    constexpr int NPART = SLICE > 1024 ? 2 : 1;
    constexpr int PB = SLICE / NPART, SP = PB / 64, PITCH = PB + 16;
    constexpr int NL = PB / 128;                            // load instructions per eight rows of a part
    static_assert(PB % 128 == 0 && PB <= 1024 && NPART * SP == KSTEPS, "slice split");
    __shared__ __align__(16) char s_stage[NW * 16 * PITCH];
    char *stage = s_stage + wave * 16 * PITCH;
    const int koff = wave * SLICE;
    int ld_row[NL], ld_col[NL];                             // (row within the eight, byte within the part) of this lane's piece
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int o = 1024 * i + 16 * lane;
        ld_row[i] = o / PB;
        ld_col[i] = o % PB;
    }
    // Neurons are dealt out in contiguous runs: workgroup q owns [q F / P, (q+1) F / P), so every
    // workgroup streams the same number of rows to within one (a row that a tile lacks costs no
    // memory traffic; 16-neuron granularity would leave an eighth of the chip idle at the end).
    // A run longer than 64 neurons (d_ff above 16384) is worked off in rounds of 64.
    // With a list the same holds for its entries (indices clamped into [0, d_ff) like the count).
    const int Fn = LIST ? min(max(p.list_n[0], 0), F) : F;
    const int j_lo_all = bat_run_lo(blk, Fn, P);
    const int j_hi_all = bat_run_lo(blk + 1, Fn, P);

    // this wave's slice of x as A-fragments: lane = (token n, k-group q)
    u32x4 xa[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (n < B) v = *reinterpret_cast<const u32x4 *>(p.x + (size_t)n * rowb + koff + (ks / SP) * PB + (q * SP + ks % SP) * 16);
        xa[ks] = v;
    }
    __syncthreads();

    auto stage_write = [&](const u32x4 (&wr)[NL], int half) {
#pragma unroll
        for (int i = 0; i < NL; ++i)
            *reinterpret_cast<u32x4 *>(stage + (8 * half + ld_row[i]) * PITCH + ld_col[i]) = wr[i];
    };
    // lanes of this wave exchange data through the tile: order the LDS traffic within the wave
    auto wave_sync = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    auto part_mma = [&](int part, f32x4 acc) {
#pragma unroll
        for (int ks = 0; ks < SP; ++ks) {
            const u32x4 frag = *reinterpret_cast<const u32x4 *>(stage + n * PITCH + (q * SP + ks) * 16);
            acc = mfma16(xa[part * SP + ks], frag, acc);
        }
        return acc;
    };
    auto part_store = [&](const f32x4 acc, int buf) {
#pragma unroll
        for (int r = 0; r < 4; ++r) s_part[buf][wave][r * 64 + lane] = acc[r];
    };
    // element (r, ln) of the 16x16 tile: token m = 4*(ln/16) + r, neuron ln%16; waves summed in order
    auto tile_sum = [&](int buf, int e) {
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += s_part[buf][w][e];
        return s;
    };
    int nlist = 0;                                          // entries of this workgroup's union list so far (uniform)
    // the token this thread compares for in the gate reduction, and its threshold (kept out of the tile loop)
    const int red_m = 4 * ((tid & 63) >> 4) + (tid >> 6);
    const float red_tau = (!DENSE && tid < 256 && red_m < B) ? p.tau[red_m] : 0.0f;
    for (int j_lo = j_lo_all; j_lo < j_hi_all; j_lo += 16 * MAX_TILES) {
    const int nown = min(16 * MAX_TILES, j_hi_all - j_lo);  // <= 64
    const int ni = (nown + 15) / 16;                        // <= MAX_TILES
    __syncthreads();                                        // the previous round is done with s_km, s_a, s_ul
    if (tid < MAX_TILES * 16) {
        s_km[tid] = 0;
        if (LIST) s_nl[tid] = tid >= nown ? 0 : min(max(p.list[j_lo + tid], 0), F - 1);
    }
    __syncthreads();

    // Every 16-neuron gate tile G_i is followed, one tile later, by the up tile U_i over the neurons of
    // G_i that at least one token keeps: G0 G1 U0 G2 U1 ... G_{ni-1} U_{ni-2} U_{ni-1}.  The rows of
    // the next tile in this order are requested while the current one is worked on, so the stream of
    // loads never drains between the gate and the up projection; U_i's rows are known by then
    // because G_i was reduced before the tile in front of U_i started.  (A single tile, ni = 1, has
    // nothing to put between G0 and U0: U0's rows are requested only after G0 is reduced.)
    // The non-gated family has gate tiles only: h is the activation itself.
    const int nseq = RELU ? ni : 2 * ni;
    auto seq_tile = [&](int sq, int &up, int &i) {
        if (RELU) { up = 0; i = sq; }
        else if (ni == 1) { up = sq; i = 0; }
        else if (sq < 2) { up = 0; i = sq; }
        else if (sq == nseq - 1) { up = 1; i = ni - 1; }
        else if (sq & 1) { up = 0; i = (sq + 1) >> 1; }
        else { up = 1; i = (sq >> 1) - 1; }
    };
    // Eight rows (half a tile) of one part of gate tile ti (up = 0: its neurons in order) or up tile ti
    // (up = 1: its union-kept neurons through the compacted list).  A row that does not exist reads
    // one shared line of zeros instead (a select on the address: no branch around any load).  up and
    // ti are uniform; the list is read whether used or not, so the loads are issued without a branch
    // on the kind of tile.
    auto rows_load = [&](u32x4 (&wr)[NL], int up, int ti, int part, int half) {
        const char *base = (up ? p.wu : p.wg) + (LIST ? (size_t)0 : (size_t)(j_lo + 16 * ti) * rowb) + koff + part * PB;
        const int lim = up ? s_ku[ti] : nown - 16 * ti;
        int lr[NL];                                         // row relative to base
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int rr = 8 * half + ld_row[i];
            const int viaList = s_ul[16 * ti + rr];
            if (LIST) lr[i] = s_nl[16 * ti + (up ? viaList & 15 : rr)];
            else lr[i] = up ? viaList : rr;
        }
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const char *src = 8 * half + ld_row[i] < lim ? base + (size_t)lr[i] * rowb + ld_col[i]
                                                         : reinterpret_cast<const char *>(k_zero16);
            wr[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src));
        }
    };
    auto gate_reduce = [&](int i, int buf) {
        if (tid < 256) {
            const int r = tid >> 6, ln = tid & 63;
            const int m = 4 * (ln >> 4) + r, nn = ln & 15, j = LIST ? s_nl[16 * i + nn] : j_lo + 16 * i + nn;
            const bool here = 16 * i + nn < nown, valid = m < B && here;
            float a = tile_sum(buf, tid);
            if (RELU) {
                if (p.b_in && valid) a += p.b_in[j];
                a = a > 0.0f ? a : (a != a ? a : 0.0f);
            } else {
                a = gate_sigma_f32(a, p.gelu);
            }
            const bool keep = valid && (DENSE ? true : (fabsf(a) >= red_tau));
            s_a[i][m][nn] = a;
            if (keep) atomicOr(&s_km[i * 16 + nn], 1 << m);
            if (p.keep && valid) p.keep[(size_t)m * F + j] = keep ? 1 : 0;
            if (RELU && here) p.hbuf[(size_t)j * 16 + m] = keep ? a : 0.0f;     // read back for union-kept neurons only
        }
    };
    // Union-kept neurons of gate tile i, compacted by ballot.  Every wave does it for itself (same
    // values to the same LDS words), so a wave only ever reads what it wrote; wave 0 appends them
    // to the workgroup's list in global memory for the down kernel.
    auto compact = [&](int i) {
        const bool mine = lane < 16 && s_km[16 * i + lane] != 0;       // never set past nown
        const unsigned long long bal = __ballot(mine);
        const int pos = __popcll(bal & ((1ull << lane) - 1ull));
        if (mine) s_ul[16 * i + pos] = lane;
        if (lane == 0) s_ku[i] = __popcll(bal);
        if (wave == 0 && mine) p.ulist[j_lo_all + nlist + pos] = LIST ? s_nl[16 * i + lane] : j_lo + 16 * i + lane;
        nlist += __popcll(bal);
        wave_sync();
    };
    auto up_reduce = [&](int i, int buf) {
        if (tid < 256) {
            const int r = tid >> 6, ln = tid & 63;
            const int m = 4 * (ln >> 4) + r, nn = ln & 15;
            if (nn < s_ku[i]) {
                const int l2 = s_ul[16 * i + nn];
                const int j = LIST ? s_nl[16 * i + l2] : j_lo + 16 * i + l2;
                const float usum = tile_sum(buf, tid);
                const bool keep = (s_km[16 * i + l2] >> m) & 1;
                p.hbuf[(size_t)j * 16 + m] = keep ? s_a[i][m][l2] * usum : 0.0f;
            }
        }
    };

    // D = X_slice * W_slice^T partial over this wave's k-slice, one tile of the sequence after the other
    u32x4 wa[NL], wb[NL];
    bool have = false;                                      // wa/wb hold the rows of the unit about to start
    int ncomp = 0;                                          // gate tiles compacted so far
    for (int sq = 0; sq < nseq; ++sq) {
        int up, ti, nup = 0, nti = 0;
        seq_tile(sq, up, ti);
        bool nready = false;                                  // the tile after this one can be requested already
        if (sq + 1 < nseq) {
            seq_tile(sq + 1, nup, nti);
            nready = !nup || nti < ncomp;
        }
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int part = 0; part < NPART; ++part) {            // unrolled: x fragments stay in registers
            if (!have) {
                rows_load(wa, up, ti, part, 0);
                rows_load(wb, up, ti, part, 1);
            }
            const bool last = part == NPART - 1;
            const bool nxt = last ? nready : true;
            const int lup = last ? nup : up, lti = last ? nti : ti, lpart = last ? 0 : part + 1;
            wave_sync();                                      // the previous part's fragment reads are done
            if (nxt) {
                stage_write(wa, 0);
                rows_load(wa, lup, lti, lpart, 0);
                stage_write(wb, 1);
                rows_load(wb, lup, lti, lpart, 1);
            } else {
                stage_write(wa, 0);
                stage_write(wb, 1);
            }
            have = nxt;
            wave_sync();
            acc = part_mma(part, acc);
        }
        part_store(acc, sq & 1);
        __syncthreads();
        if (!up) {
            gate_reduce(ti, sq & 1);
            __syncthreads();                                  // the tile's keep masks are complete
            compact(ti);
            ++ncomp;
        } else {
            up_reduce(ti, sq & 1);
        }
    }
    }   // rounds
    if (tid == 0) p.ucnt[blk] = nlist;
}

constexpr int DN_COLS = 256;                    // columns per workgroup in kernel B
constexpr int DN_SUB = 128;                     // columns staged per pass
constexpr int DN_PITCH = DN_SUB * 2 + 32;       // LDS row pitch (bytes): 4 rows of a transpose read hit distinct banks
constexpr int DN_TILE_BYTES = 32 * DN_PITCH;    // one wave's staging tile: 32 neurons x 128 columns
constexpr int DN_MAX_ROWS = 2048;               // union neurons per row group
constexpr int DN_MAX_WGS = 64;                  // gate/up workgroups per row group

__global__ void __launch_bounds__(512, 4)
k_bat_down(const BatParams p)
{
    extern __shared__ __align__(16) unsigned char smem_dn[];
    unsigned char *s_tile = smem_dn;                                    // [8][DN_TILE_BYTES], later the fold buffers
    int *s_rows = reinterpret_cast<int *>(smem_dn + 8 * DN_TILE_BYTES); // [DN_MAX_ROWS]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroups go to the 8 XCDs round-robin by id, and each XCD has its own L2.  The column groups of
    // one row group all read the same h lines and row list, so they are given ids of one residue
    // class mod 8 where the grid divides evenly: an h line then crosses the fabric once, not 8 times.
    int wg = blockIdx.x;
    if (gridDim.x % 8 == 0) wg = (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
    const int cg = wg % p.CG, rg = wg / p.CG;
    const int d = p.d, F = p.F, B = p.B;
    const size_t rowb = (size_t)d * 2;
    const int col0 = cg * DN_COLS;

    // ---- this row group's neurons = those of the gate/up workgroups [w0, w1): their union lists, laid end
    // to end (ascending).  The list entries are requested before the counts are known; an entry past
    // its workgroup's count is stale memory inside the list array and is dropped.
    const int w0 = (int)((long long)rg * p.P / p.RG), w1 = (int)((long long)(rg + 1) * p.P / p.RG);
    const int nw = w1 - w0;                                             // <= DN_MAX_WGS (host check)
    const int Fn = p.list ? min(max(p.list_n[0], 0), F) : F;
    auto run_lo = [&](int w) { return bat_run_lo(w, Fn, p.P); };
    const int cnt_l = lane < nw ? p.ucnt[w0 + lane] : 0;               // every wave: the counts, one per lane
    constexpr int PRE = 4;                                              // entries per thread held in registers
    int pre_v[PRE];
#pragma unroll
    for (int k = 0; k < PRE; ++k) {
        const int w = wave + 8 * k;
        const int jj = w < nw ? run_lo(w0 + w) + lane : F;
        pre_v[k] = jj < F ? p.ulist[jj] : 0;
    }
    int inc = cnt_l;                                                    // inclusive scan over the lanes
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    const int exc = inc - cnt_l;
    const int nrows = __shfl(inc, 63);                                  // <= DN_MAX_ROWS (host check)
#pragma unroll
    for (int k = 0; k < PRE; ++k) {
        const int w = wave + 8 * k, ws = w < nw ? w : 0;
        const int c = __shfl(cnt_l, ws), o = __shfl(exc, ws);
        if (w < nw && lane < c) s_rows[o + lane] = pre_v[k];
    }
    // whatever the registers did not cover: more than 8 * PRE workgroups, or lists longer than 64
    for (int w = wave; w < nw; w += 8) {
        const int c = __shfl(cnt_l, w), o = __shfl(exc, w);
        for (int e = (w < 8 * PRE ? 64 : 0) + lane; e < c; e += 64) s_rows[o + e] = p.ulist[run_lo(w0 + w) + e];
    }
    __syncthreads();

    // Wave w works on column half sub = w & 1 of the workgroup's 256 columns and on the 32-neuron
    // blocks rw, rw + 4, ... (rw = w >> 1): units of 32 rows x 128 columns dealt round-robin, so the
    // eight waves differ by at most one unit.
    const int sub = wave & 1, rw = wave >> 1;
    f32x4 acc[DN_SUB / 16];
#pragma unroll
    for (int t = 0; t < DN_SUB / 16; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int n = lane & 15, q = lane >> 4;
    unsigned char *tile = s_tile + wave * DN_TILE_BYTES;
    const int nkb = (nrows + 31) / 32;
    static_assert(DN_COLS == 2 * DN_SUB, "two staging passes per block of neurons");

    // h[token n][8 consecutive list entries] of block kb (raw fp32, converted when used)
    auto h_load = [&](float (&hv)[8], int kb) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int e = 32 * kb + 8 * q + i;
            hv[i] = (e < nrows && n < B) ? p.hbuf[(size_t)s_rows[e] * 16 + n] : 0.0f;
        }
    };
    // W_down[32 list entries][128 columns]: half-waves read 256-byte row pieces
    auto w_load = [&](u32x4 (&wv)[8], int kb) {
#pragma unroll
        for (int ii = 0; ii < 8; ++ii) {
            const int c = lane + 64 * ii, row = c >> 4, cc = c & 15;
            const int e = 32 * kb + row;
            const int col = col0 + sub * DN_SUB + 8 * cc;
            // rows past the list repeat the last row (their h is zero); columns past d cannot
            // occur for the supported widths (d is a multiple of 256)
            const int er = e < nrows ? e : nrows - 1;
            wv[ii] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p.wd + (size_t)s_rows[er] * rowb + (size_t)col * 2));
        }
    };
    auto process = [&](const u32x4 (&wv)[8], const u32x4 ahi, const u32x4 alo) {
#pragma unroll
        for (int ii = 0; ii < 8; ++ii) {
            const int c = lane + 64 * ii, row = c >> 4, cc = c & 15;
            *reinterpret_cast<u32x4 *>(tile + row * DN_PITCH + cc * 16) = wv[ii];
        }
        // K-major B-fragments by transpose reads: in each 16-lane group lane t = 4r + c4 supplies
        // row 8q + r, columns 4*c4 .. 4*c4+3 and receives column t of rows 8q .. 8q+3
        const int r = (lane & 15) >> 2, c4 = lane & 3;
#pragma unroll
        for (int t = 0; t < DN_SUB / 16; ++t) {
            const unsigned char *src = tile + (8 * q + r) * DN_PITCH + (t * 16 + 4 * c4) * 2;
            const s16x4 b0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)src);
            const s16x4 b1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(src + 4 * DN_PITCH));
            const uint2 u0 = __builtin_bit_cast(uint2, b0), u1 = __builtin_bit_cast(uint2, b1);
            const u32x4 bf = {u0.x, u0.y, u1.x, u1.y};
            acc[t] = mfma16(ahi, bf, acc[t]);
            acc[t] = mfma16(alo, bf, acc[t]);
        }
    };
    auto split_h = [&](const float (&hv)[8], u32x4 &ahi, u32x4 &alo) {
        unsigned int hi16[8], lo16[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            hi16[i] = f32_to_bf16_bits(hv[i]);
            lo16[i] = f32_to_bf16_bits(hv[i] - __uint_as_float(hi16[i] << 16));
        }
        ahi = u32x4{hi16[0] | (hi16[1] << 16), hi16[2] | (hi16[3] << 16), hi16[4] | (hi16[5] << 16), hi16[6] | (hi16[7] << 16)};
        alo = u32x4{lo16[0] | (lo16[1] << 16), lo16[2] | (lo16[3] << 16), lo16[4] | (lo16[5] << 16), lo16[6] | (lo16[7] << 16)};
    };

    // A unit is requested and consumed in turn; the waves of two workgroups share a compute unit (at most 128
    // registers per lane, 80 KiB of LDS each), and it is their loads that cover this wave's consumption.
    // (Requesting the next unit before consuming the current one needed 182 registers, one workgroup per
    // compute unit, and was 1.5 - 4 % slower per step, most with a sparse union.)
    u32x4 wA[8];
    float hA[8];
    for (int kb = rw; kb < nkb; kb += 4) {
        u32x4 ahi, alo;
        h_load(hA, kb);
        w_load(wA, kb);
        split_h(hA, ahi, alo);
        process(wA, ahi, alo);
    }

    // ---- fixed-order fold of the four row-waves of each column half through LDS, then the partial
    // y of this row group
    __syncthreads();
    float *s_red = reinterpret_cast<float *>(s_tile);                   // [2 halves][2][8 tiles][4][64]
    constexpr int ACC_FLOATS = (DN_SUB / 16) * 4 * 64;
#pragma unroll
    for (int s2 = 2; s2 >= 1; s2 >>= 1) {
        if (rw >= s2 && rw < 2 * s2) {
            float *dst = s_red + (size_t)(sub * 2 + (rw - s2)) * ACC_FLOATS;
#pragma unroll
            for (int t = 0; t < DN_SUB / 16; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) dst[(t * 4 + r) * 64 + lane] = acc[t][r];
        }
        __syncthreads();
        if (rw < s2) {
            const float *src = s_red + (size_t)(sub * 2 + rw) * ACC_FLOATS;
#pragma unroll
            for (int t = 0; t < DN_SUB / 16; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[t][r] += src[(t * 4 + r) * 64 + lane];
        }
        __syncthreads();
    }
    if (rw == 0) {
#pragma unroll
        for (int t = 0; t < DN_SUB / 16; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = 4 * q + r, col = col0 + sub * DN_SUB + t * 16 + n;
                if (m < B && col < d) p.partial[((size_t)rg * B + m) * d + col] = acc[t][r];
            }
    }
}

}  // namespace

size_t clada_ws_decode_batched(int32_t d_ff)
{
    return align_up(sizeof(float) * 16 * (size_t)d_ff, 256) + align_up(sizeof(int) * (size_t)d_ff, 256) +
           align_up(sizeof(int) * COOP_MAX_WGS, 256);
}

// Launch shape of the batched path for a layer and a pass of B tokens; false when the shape is not eligible
// (decided by dtype and sizes alone, before anything is launched).
static bool bat_plan(const clada_ctx *ctx, const clada_layer *layer, int B, int *P_out, int *CG_out, int *RG_out)
{
    const int d = layer->d, F = layer->d_ff;
    if (layer->dtype != CLADA_BF16 || B < 2 || B > 16) return false;
    const int ksteps = d / 256;                                  // 8 waves x ksteps x 32 = d (5 waves x 16 or 32 x 32 for ksteps 10, 20)
    if (d % 256 != 0 || !(ksteps == 4 || ksteps == 8 || ksteps == 10 || ksteps == 12 || ksteps == 16 || ksteps == 20 ||
                          ksteps == 24 || ksteps == 32))
        return false;
    const int P = ctx->num_cu < COOP_MAX_WGS ? ctx->num_cu : COOP_MAX_WGS;
    const int CG = (d + DN_COLS - 1) / DN_COLS;
    int RG = P / CG;
    if (RG < 1) RG = 1;
    if (RG > 64) RG = 64;
    if (RG > 1 && (CG * RG) % 8 != 0 && (CG * (RG - 1)) % 8 == 0) --RG;     // a grid the XCD-aware map of the down kernel divides
    // row group rg = the neurons of the gate/up workgroups [rg P / RG, (rg+1) P / RG)
    auto group_fits = [&](int rgs) {
        if (rgs > P) return false;
        for (int rg = 0; rg < rgs; ++rg) {
            const int w0 = (int)((long long)rg * P / rgs), w1 = (int)((long long)(rg + 1) * P / rgs);
            if (w1 - w0 > DN_MAX_WGS || bat_run_lo(w1, F, P) - bat_run_lo(w0, F, P) > DN_MAX_ROWS) return false;
        }
        return true;
    };
    while (!group_fits(RG) && RG < 64) RG *= 2;                         // wide layers: more, smaller row groups
    if (!group_fits(RG)) return false;
    *P_out = P; *CG_out = CG; *RG_out = RG;
    return true;
}

bool clada_decode_batched_eligible(const clada_ctx *ctx, const clada_layer *layer, int32_t B)
{
    int P, CG, RG;
    return bat_plan(ctx, layer, B, &P, &CG, &RG);
}

// Bytes of partial outputs one pass of the batched path writes at most: [RG <= 64][B <= 16][d] fp32.
size_t clada_ws_decode_batched_partial(int32_t d)
{
    return align_up(sizeof(float) * 64 * 16 * (size_t)d, 256);
}

// Runs the batched MFMA path when the shape is eligible (*ran; an ineligible shape launches nothing and the
// caller uses the generic kernels).
clada_status clada_decode_batched(clada_ctx *ctx, const clada_layer *layer, const void *x, int32_t B,
                                  const float *tau, void *y, unsigned char *keep, float *partial,
                                  char *scratch, bool dense, hipStream_t stream, bool *ran,
                                  const int32_t *list, const int32_t *list_n)
{
    *ran = false;
    const int d = layer->d, F = layer->d_ff;
    int P, CG, RG;
    if (!bat_plan(ctx, layer, B, &P, &CG, &RG)) return CLADA_OK;

    BatParams p;
    p.wg = (const char *)layer->w_gate; p.wu = (const char *)layer->w_up; p.wd = (const char *)layer->w_down;
    p.x = (const char *)x; p.tau = tau;
    p.hbuf = reinterpret_cast<float *>(scratch);
    p.ulist = reinterpret_cast<int *>(scratch + align_up(sizeof(float) * 16 * (size_t)F, 256));
    p.ucnt = reinterpret_cast<int *>(scratch + align_up(sizeof(float) * 16 * (size_t)F, 256) + align_up(sizeof(int) * (size_t)F, 256));
    p.keep = keep; p.partial = partial;
    p.d = d; p.F = F; p.B = B; p.P = P; p.RG = RG; p.CG = CG;
    p.gelu = layer->kind == CLADA_FFN_GEGLU ? 1 : 0;
    const bool relu = layer->kind == CLADA_FFN_RELU;
    p.b_in = layer->b_in;
    p.list = list; p.list_n = list_n;

#define CLADA_BAT_LAUNCH(KS, NW, RELU)                                                                                    \
    {                                                                                                                      \
        if (list)       hipLaunchKernelGGL((k_bat_gateup<KS, NW, true, true, RELU>), dim3(P), dim3(NW * 64), 0, stream, p);   \
        else if (dense) hipLaunchKernelGGL((k_bat_gateup<KS, NW, true, false, RELU>), dim3(P), dim3(NW * 64), 0, stream, p);  \
        else            hipLaunchKernelGGL((k_bat_gateup<KS, NW, false, false, RELU>), dim3(P), dim3(NW * 64), 0, stream, p); \
    }
#define CLADA_BAT_CASE(D, KS, NW)                                                                            \
    if (d == D) {                                                                                             \
        static_assert(D == NW * 32 * KS, "waves x k-steps x 32 = d");                                         \
        if (relu) CLADA_BAT_LAUNCH(KS, NW, true) else CLADA_BAT_LAUNCH(KS, NW, false)                         \
    }
    CLADA_BAT_CASE(1024, 4, 8) CLADA_BAT_CASE(2048, 8, 8) CLADA_BAT_CASE(2560, 16, 5) CLADA_BAT_CASE(3072, 12, 8)
    CLADA_BAT_CASE(4096, 16, 8) CLADA_BAT_CASE(5120, 32, 5) CLADA_BAT_CASE(6144, 24, 8) CLADA_BAT_CASE(8192, 32, 8)
#undef CLADA_BAT_LAUNCH
#undef CLADA_BAT_CASE
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    const size_t lds = 8 * (size_t)DN_TILE_BYTES + sizeof(int) * DN_MAX_ROWS;
    static std::atomic<bool> attr_set{false};                           // set once per process (two first callers may both set it)
    if (!attr_set.load(std::memory_order_relaxed)) {
        CLADA_CHECK_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(k_bat_down),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set.store(true, std::memory_order_relaxed);
    }
    hipLaunchKernelGGL(k_bat_down, dim3(CG * RG), dim3(512), lds, stream, p);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    clada_launch_finalize(2, partial, RG, B, d, (char *)y, stream, relu ? layer->b_out : nullptr);
    CLADA_CHECK_HIP(ctx, hipGetLastError());
    *ran = true;
    return CLADA_OK;
}
