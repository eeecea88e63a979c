/*
 * clada.h -- C ABI of the MI355X (gfx950) implementation of CLADA's decode-time
 * hot path: the thresholded sparse SwiGLU FFN and the small calls that feed it
 * (arXiv 2502.19078, section 3.2 "Dynamic Threshold Strategy" and the
 * algorithm "CLADA Inference").
 *
 * General rules
 *   - Every tensor pointer is BORROWED DEVICE memory owned by the caller; it
 *     must stay valid until the work enqueued by the call has finished.  The
 *     only host pointers are the context, the small descriptor structs and the
 *     scalars.  `hip_stream` is a hipStream_t passed as void* (NULL = the
 *     default stream).
 *   - Calls validate their arguments on the host before touching HIP, enqueue
 *     kernels on `hip_stream` and return without synchronising.  They allocate
 *     nothing: scratch lives in the context's workspace, sized at
 *     clada_create() with clada_workspace_bytes().
 *   - A context serves one stream at a time; calls issued to one context from
 *     several threads or streams at once race on its workspace.
 *   - Every call returns a clada_status and never throws or aborts;
 *     clada_last_error() gives the text of the last failure of that context.
 *   - Weights are neuron-major: W_gate[d_ff][d], W_up[d_ff][d], W_down[d_ff][d],
 *     row-major, row j holding neuron j's two input-projection rows and its
 *     output-projection column (text under the neuron-activation equation of
 *     section 3.2.1).  Rows must be 16-byte aligned: d*sizeof(elem) % 16 == 0.
 *   - Activations x/y use the layer's dtype; statistics, signals, thresholds
 *     are fp32; indices are int32.
 */
#ifndef CLADA_H
#define CLADA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct clada_ctx clada_ctx; /* opaque; owns only its workspace */

typedef enum {
    CLADA_OK = 0,
    CLADA_ERR_NULL = 1,      /* a required pointer is NULL */
    CLADA_ERR_SHAPE = 2,     /* a size is non-positive, too large, or violates a divisibility rule */
    CLADA_ERR_DTYPE = 3,     /* unknown clada_dtype */
    CLADA_ERR_ALIGN = 4,     /* a pointer is not 16-byte aligned */
    CLADA_ERR_WORKSPACE = 5, /* the context's workspace is too small for this call */
    CLADA_ERR_VALUE = 6,     /* a scalar argument is out of its domain */
    CLADA_ERR_HIP = 7        /* a HIP runtime call failed (text in clada_last_error) */
} clada_status;

typedef enum { CLADA_F32 = 0, CLADA_BF16 = 1 } clada_dtype;

/* Limits checked by every call (CLADA_ERR_SHAPE beyond them). */
#define CLADA_MAX_D 8192       /* model width d; also d*sizeof(elem) <= 16384 */
#define CLADA_MAX_DFF 262144   /* FFN width d_ff           */
#define CLADA_MAX_BATCH 64     /* decode batch B           */
#define CLADA_MAX_LAYERS 4096  /* layers L in clada_threshold */

/* Context.  workspace_bytes == 0 creates a context that touches no GPU (every
 * compute call then fails with CLADA_ERR_WORKSPACE after validation); otherwise
 * the workspace is allocated on device `device_id`, which must be the device
 * the caller's tensors and stream live on. */
clada_status clada_create(clada_ctx **out, int device_id, size_t workspace_bytes);
void clada_destroy(clada_ctx *ctx);
const char *clada_status_str(int32_t s);   /* s: a clada_status; any other value gives "CLADA_ERR_UNKNOWN" */
const char *clada_last_error(const clada_ctx *ctx);

/* Launch-shape tuning knobs; results never depend on them beyond fp32 summation
 * order.  Names: "decode.b1" (batch-1 decode kernel: 1 = split-d kernel, with
 * cross-workgroup load balancing where the layer is large enough for it to pay
 * [default], 2 = split-d kernel without balancing, 3 = with balancing whenever
 * the launch allows it, 0 = the generic kernels), "decode.own_first" (1..14, neurons a
 * workgroup keeps for itself before the balanced hand-over; 0 = default),
 * "decode.wgs_per_cu" (1 or 2 workgroups per compute unit for the generic kernel),
 * "decode.stack" (how the whole-stack calls run: 3 = lanes [default], 2 = chained
 * launches, 1 = one persistent kernel for all layers where the shape has one, 0 = the L
 * per-layer calls; see clada_sparse_ffn_stack_decode), "decode.lane_occ2" (1 = the lanes of
 * batch-1 stacks with rows of 4, 5 or 8 KiB use the kernel instance of which two workgroups
 * fit a compute unit [default], 0 = the instance of the per-layer call),
 * "decode.batched" (1 = matrix-core kernels for bf16 batches of 2 and more, 16 tokens
 * per pass [default], 0 = the
 * generic kernels), "decode.spin_limit" (how often a balanced batch-1 kernel polls
 * for the other workgroups' masks before it gives up; default 4096, a few
 * milliseconds against the microseconds a healthy exchange takes;
 * 0 = give up without polling; see clada_device_fault), "prefix.tile" (workgroup
 * tiles of the bf16 prefill GEMMs: 1 = 128 tokens, 2 = 256 tokens wherever the shape
 * allows, 0 = chosen by shape [default]), "diag.kernel_events" (1 = every decode call also
 * records HIP events around its kernels for clada_diag_kernel_times; default 0).
 * Unknown names or out-of-range values give CLADA_ERR_VALUE and change nothing. */
clada_status clada_set_option(clada_ctx *ctx, const char *name, int32_t value);

/* The balanced batch-1 decode kernel waits, inside the kernel, for the keep masks of
 * all its workgroups, one per compute unit.  They can only stay away while something
 * else holds compute units they need: ANY kernel that runs at the same time on another
 * stream, context or process and fills whole compute units can do that (a second
 * balanced call, but also e.g. an attention kernel of the caller's own model).  A caller
 * that overlaps other GPU work with the FFN calls should set option "decode.b1" = 2
 * (no cross-workgroup wait anywhere).  The wait is bounded: past the limit the kernel
 * gives up, the call's output and every later output of the context is NaN, and this
 * call (which synchronises the device) reports *fault_out = 1.  A context that has
 * faulted must be destroyed. */
clada_status clada_device_fault(clada_ctx *ctx, int32_t *fault_out);

/* Upper bound of the workspace any call needs for these sizes.  Pass 0 for a
 * size whose call will not be used (T for prefix_stats/calibrate/the CETT calls, V for
 * cognitive_signals, B for the decode calls). */
size_t clada_workspace_bytes(int32_t d, int32_t d_ff, int32_t B, int32_t T, int32_t V);

/* FFN family.  CLADA_FFN_SWIGLU (0, the default of a zeroed struct): the gated
 * SiLU FFN of the LLaMA / Mistral models, sigma = SiLU in the neuron-activation
 * equation of section 3.2.1.  CLADA_FFN_RELU: the non-gated FFN of the OPT models
 * the paper also evaluates -- no V_in factor, sigma = ReLU, biases:
 *   a_bj = max(0, W_in[j,:] . x_b + b_in[j]),  keep_bj = a_bj >= tau_final[b],
 *   y_b = sum_{j kept} a_bj W_out[j,:] + b_out.
 * For it w_gate holds W_in [d_ff][d], w_down holds W_out neuron-major [d_ff][d]
 * (HF fc2.weight transposed), w_up is ignored; b_in [d_ff] and b_out [d] are fp32
 * device arrays or NULL (zero).  Supported by every entry point; in the CETT calls
 * n_j(x) = a_j W_out[j,:] and MLP(x) = sum_j n_j(x) + b_out (the bias is the layer's,
 * not a neuron's: it enters the denominator only).
 * CLADA_FFN_GEGLU: the gated FFN of the Gemma model the paper also evaluates -- as
 * CLADA_FFN_SWIGLU in every respect (three matrices, no biases, every entry point)
 * except sigma = GELU in its tanh form,
 *   sigma(g) = g/2 (1 + tanh(sqrt(2/pi) (g + 0.044715 g^3))). */
typedef enum { CLADA_FFN_SWIGLU = 0, CLADA_FFN_RELU = 1, CLADA_FFN_GEGLU = 2 } clada_ffn_kind;

typedef struct {
    const void *w_gate, *w_up, *w_down; /* device, each [d_ff][d] neuron-major */
    int32_t d, d_ff;
    int32_t dtype;                      /* a clada_dtype; an unknown value is CLADA_ERR_DTYPE */
    int32_t kind;                       /* a clada_ffn_kind; an unknown value is CLADA_ERR_VALUE */
    const float *b_in, *b_out;          /* CLADA_FFN_RELU only */
} clada_layer;

typedef struct {            /* device outputs, caller-allocated; any may be NULL to skip */
    float *sum_abs_act;     /* [d_ff]  sum_t |a_tj|                                   */
    float *sum_sq_act;      /* [d_ff]  sum_t a_tj^2                                   */
    float *max_abs_act;     /* [d_ff]  max_t |a_tj|                                   */
    float *sum_sq_h;        /* [d_ff]  sum_t h_tj^2,  h = a * u                        */
    float *A;               /* [d_ff]  neuron activation magnitude A_j (section 3.2.1) */
    float *abs_act_pool;    /* [T][d_ff]  |a_tj|, the pool the base threshold is a quantile of */
} clada_prefix_out;

/* Prefill statistics (section 3.2.1 "Neuron Activation Prefilling"; algorithm
 * "CLADA Inference", prefill phase).  Dense SwiGLU FFN over the prefix
 * x [T][d]:  a = SiLU(x W_gate^T), h = a .* (x W_up^T), y = h W_down, and the
 * per-neuron aggregates of clada_prefix_out, with
 *   A_j = || h_{:,j} W_down[j,:] ||_F = sqrt(sum_t h_tj^2) * ||W_down[j,:]||_2.
 * y [T][d] (layer dtype) may be NULL.  T >= 1.  bf16 layers use bf16 MFMA with
 * fp32 accumulation (h is rounded to bf16 before the down projection); fp32
 * layers use fp32 MFMA. */
clada_status clada_prefix_stats(clada_ctx *ctx, const clada_layer *layer, const void *x,
                                int32_t T, void *y, const clada_prefix_out *out,
                                void *hip_stream);

/* Base threshold from the pooled prefix magnitudes: the nearest-rank
 * q-quantile, i.e. the k-th smallest of abs_act_pool[0..n), k = max(1,
 * ceil(q*n)) taken in fp64.  This is the percentile stand-in for the
 * error-bounded threshold search of section 3.2.2.  Values must be
 * non-negative finite floats (or +inf); NaN entries make the result
 * unspecified.  q in [0,1), n >= 1.  Result: one fp32 on the device. */
clada_status clada_threshold_calibrate(clada_ctx *ctx, const float *abs_act_pool, int64_t n,
                                       float target_sparsity, float *tau_base_out,
                                       void *hip_stream);

/* Error-bounded base threshold (section 3.2.2, base-threshold equation):
 *   tau_base = max eps  subject to  mean_t CETT(x_t; eps) <= bound   (the paper uses 0.2),
 *   CETT(x; eps) = || sum_{j : |a_j(x)| < eps} h_j(x) W_down[j,:] ||_2 / || MLP(x) ||_2
 * over the validation tokens x_val [T][d] (layer dtype), with a, h as in
 * clada_prefix_stats; the cut rule (strict '<' on |SiLU(gate)|, NaN never cut)
 * is the decode call's, so the result feeds clada_threshold directly.  A token
 * whose dense output is zero counts as CETT = 0.
 * The search bisects the bit pattern of eps between 0 (cuts nothing) and +inf
 * (cuts everything) with the bracket on the device: n_probes in [1,31] probes,
 * each one masked down projection; 31 resolve the float exactly, fewer return
 * the lower, feasible end of the remaining bracket.  Where the mean is not
 * monotone in eps at the scale of single neurons the result is a boundary of
 * the feasible set, not necessarily its last one.  bound in [0,1).
 * Outputs (device): tau_base_out [1]; mean_cett_out [1] = the mean at
 * tau_base_out, or NULL.  bf16 layers round h to bf16 before the projections. */
clada_status clada_threshold_search_cett(clada_ctx *ctx, const clada_layer *layer, const void *x_val,
                                         int32_t T, float bound, int32_t n_probes,
                                         float *tau_base_out, float *mean_cett_out, void *hip_stream);

/* The quantity the search bounds, at one given eps (host scalar; +inf allowed,
 * NaN is CLADA_ERR_VALUE): cett_out [T] per validation token and/or mean_out [1]
 * (device; one of them may be NULL). */
clada_status clada_cett_eval(clada_ctx *ctx, const clada_layer *layer, const void *x_val, int32_t T,
                             float eps, float *cett_out, float *mean_out, void *hip_stream);

/* Cognitive-load signals (section 2.3.1, surprisal and entropy equations), per
 * row b of logits [B][V] (logits_dtype: a clada_dtype, fp32 or bf16), natural log:
 *   surprisal[b] = -log softmax(z_b)[token_ids[b]],  entropy[b] = -sum_v p_v log p_v.
 * One pass over the logits (online log-sum-exp).  A row holding NaN or +inf, or
 * only -inf, yields NaN for both; a token id outside [0,V) yields NaN surprisal.
 * These are device-side values: no status is raised for them. */
clada_status clada_cognitive_signals(clada_ctx *ctx, const void *logits,
                                     int32_t logits_dtype, int32_t B, int32_t V,
                                     const int32_t *token_ids, float *surprisal,
                                     float *entropy, void *hip_stream);

/* Token-aware threshold (section 3.2.3, final-threshold equation):
 *   tau_final[l][b] = tau_base[l] * (1 + lambda[l]*[s_b > tau_s] + gamma[l]*[H_b > tau_H]).
 * Strict '>', signed coefficients, no clamping.  tau_s / tau_H may be +-inf to
 * force the indicators off / on.  All arrays on the device. */
clada_status clada_threshold(clada_ctx *ctx, const float *tau_base, const float *lambda,
                             const float *gamma, int32_t L, const float *surprisal,
                             const float *entropy, int32_t B, float tau_s, float tau_H,
                             float *tau_final, void *hip_stream);

/* The two calls above as one launch (the generation phase of the algorithm "CLADA
 * Inference" computes the signals and then the thresholds once per token, ahead of
 * the layers): surprisal / entropy [B] as clada_cognitive_signals writes them, and
 * tau_final [L][B] as clada_threshold would compute it from them -- the block that
 * finishes a row of logits also writes that row's L thresholds.  Same arguments,
 * same limits, same results bit for bit. */
clada_status clada_signals_threshold(clada_ctx *ctx, const void *logits, int32_t logits_dtype,
                                     int32_t B, int32_t V, const int32_t *token_ids,
                                     const float *tau_base, const float *lambda, const float *gamma,
                                     int32_t L, float tau_s, float tau_H, float *surprisal,
                                     float *entropy, float *tau_final, void *hip_stream);

/* clada_cognitive_signals for callers that cannot allocate device memory at all, not
 * even a context's workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results bit for bit, but the
 * kernel's scratch (block partials and arrival counters) is a fixed array inside the
 * library's device code, about 256 KiB on every GPU the library runs on, held until the
 * process ends; the call makes no hipMalloc / hipFree and uses no workspace, so `ctx`
 * may be a context created with workspace_bytes == 0 (it only carries the error text).
 * The device the stream and the tensors live on must be the current one (hipSetDevice).
 * V above CLADA_STATIC_SIGNALS_MAX_V is rejected with CLADA_ERR_SHAPE.  The first call
 * on a device looks the array's address up (make it outside a graph capture).  All
 * calls on one GPU share the array: calls that overlap on one GPU (two streams, two
 * threads) race on it -- issue them on one stream. */
#define CLADA_STATIC_SIGNALS_MAX_V (1 << 20)
clada_status clada_cognitive_signals_static(clada_ctx *ctx, const void *logits, int32_t logits_dtype,
                                            int32_t B, int32_t V, const int32_t *token_ids,
                                            float *surprisal, float *entropy, void *hip_stream);

/* Thresholded sparse SwiGLU FFN for one layer at decode time (algorithm "CLADA
 * Inference", generation phase: regenerate the mask by thresholding, then the
 * sparse forward pass).  For each token b of x [B][d]:
 *   a_bj = SiLU(W_gate[j,:] . x_b)          (dense gate projection, fp32 accumulate)
 *   keep_bj = |a_bj| >= tau_final[b]        (fp32 compare; NaN is cut)
 *   y_b = sum_{j kept} a_bj (W_up[j,:] . x_b) W_down[j,:]
 * Only rows of W_up / W_down of neurons kept by at least one token are read.
 * tau_final [B] is this layer's row of clada_threshold's output.
 * Optional outputs (NULL to skip): active_idx [d_ff] ascending indices of the
 * union of kept neurons (entries past the count are left untouched);
 * n_active [1+B] = {union count, per-token counts}; mask_bits
 * [B][ceil(d_ff/32)] bit j%32 of word j/32 set iff keep_bj.
 * The result is bit-reproducible from run to run (fixed summation order).
 * Paths: B = 1 with rows of whole KiB runs the row-streaming kernel (vector ALUs); bf16
 * batches of 2 and more run on the matrix cores, 16 tokens per pass, every weight row read
 * once per pass.  Everything else -- fp32 batches in particular -- runs a generic kernel
 * that works through the tokens one by one and reads the kept rows once PER TOKEN: correct
 * and tested, but its HBM traffic grows with B (a limit of this library, not of the method). */
clada_status clada_sparse_ffn_decode(clada_ctx *ctx, const clada_layer *layer, const void *x,
                                     int32_t B, const float *tau_final, void *y,
                                     int32_t *active_idx, int32_t *n_active,
                                     uint32_t *mask_bits, void *hip_stream);

/* Dense twin of clada_sparse_ffn_decode (every neuron kept; the paper's "Dense"
 * column): same layout and reduction order, gate/up/down rows all read. */
clada_status clada_dense_ffn_decode(clada_ctx *ctx, const clada_layer *layer, const void *x,
                                    int32_t B, void *y, void *hip_stream);

/* The L sparse FFN calls of one decode step as ONE call, for stacks whose layers are
 * independent problems: layer l has its own input row x[l] and its own output row y[l]
 * (the FFN-stack workloads this library is measured on; in a model whose next layer
 * consumes y[l] through attention the per-layer call above is the one that applies).
 * Mask compression and "whole-stack persistence" are what the paper's limitations and
 * future-work paragraphs leave open; this is the second.  Knowing the whole stack, the
 * library can hide what every per-layer call pays: the start-up of a kernel, its ragged
 * end, and the launch of the final reduction.  Option "decode.stack" chooses how:
 *   3 (default)  lanes: the layers go round two or three streams -- hip_stream and streams
 *                that the context owns (default priority), forked and joined by events
 *                inside the call.  To the caller the call is ordered on hip_stream like any
 *                other, and a stream capture of hip_stream records all lanes.  The compute
 *                units that layer l has released run layer l+1 already; where the kernel
 *                has an instance of which two workgroups fit a compute unit (rows of 4, 5
 *                and 8 KiB), workgroups of different layers share every unit.  The lanes use
 *                the kernels without cross-workgroup balancing (kernels that wait for
 *                their own workgroups must not share the chip).
 *   2            chained launches on hip_stream: the kernel of layer l also sums the
 *                partial outputs of layer l-1; one reduction launch per call.
 *   1            one persistent kernel walks the layers (bf16 rows of 4, 5, 8 or 10 KiB,
 *                all workgroups resident at once); measured slower for sparse stacks.
 *   0            the L per-layer calls, issued by the library.
 *   layers [L] (host array; all of one d, d_ff, dtype and kind), x [L][B][d], y [L][B][d]
 *   (layer dtype), tau_final [L][B] (clada_threshold's output), 1 <= B <= 64, n_active
 *   [L][1 + B] or NULL (per layer, the layout of the per-layer call).
 * Results are bit-identical to L calls of clada_sparse_ffn_decode with the same balancing
 * (modes 0 - 2: the context's "decode.b1"; mode 3: as with "decode.b1" = 2): the same
 * kernels' order of summation.  For B = 1, modes 2 and 3 need the batch-1 kernel's shapes
 * (rows of whole KiB), 256 compute units or more and n_active = NULL.  For B >= 2 there is
 * mode 3 only: the units (layer, pass of up to 16 tokens) of the matrix-core path go round
 * three lanes, where that path applies (bf16, its widths) and n_active = NULL.  Every mode
 * falls back to mode 0 where it does not apply.  The remarks on clada_device_fault apply to modes 0 - 2
 * (balanced kernels wait, bounded, for their own workgroups).  A context serves one call
 * at a time, on whatever stream.  The first call in mode 3 creates the context's lane streams
 * and events: make it before hip_stream is captured.  clada_dense_ffn_stack_decode is the
 * dense twin. */
clada_status clada_sparse_ffn_stack_decode(clada_ctx *ctx, const clada_layer *layers, int32_t L,
                                           const void *x, int32_t B, const float *tau_final, void *y,
                                           int32_t *n_active, void *hip_stream);
clada_status clada_dense_ffn_stack_decode(clada_ctx *ctx, const clada_layer *layers, int32_t L,
                                          const void *x, int32_t B, void *y, void *hip_stream);

/* Prefix-static masks.  The generation phase of the algorithm "CLADA Inference"
 * says the masks are regenerated "by thresholding A": read literally, the
 * prefill magnitudes A_j (clada_prefix_out.A, neuron-activation equation of
 * section 3.2.1) are compared with tau_final, so a layer has one mask per
 * indicator pattern and the gate rows of cut neurons are never read.
 *   clada_static_mask_threshold: active_idx = ascending { j : A[j] >= tau_final[0] }
 *     (cut iff strictly below; NaN is cut), n_active[0] = its size.
 *   clada_static_mask_topk: the k neurons with the largest score (hard top-k on a
 *     prefix aggregate, how section 4 characterises the Griffin baseline); equal
 *     scores go to the lower index, NaN ranks below every number; ascending
 *     indices, n_active[0] = k.  0 <= k <= d_ff.
 * A / score [d_ff] fp32, tau_final [1] fp32, active_idx [d_ff] int32 (entries past
 * the count untouched), n_active [1] int32: all device. */
clada_status clada_static_mask_threshold(clada_ctx *ctx, const float *A, int32_t d_ff,
                                         const float *tau_final, int32_t *active_idx,
                                         int32_t *n_active, void *hip_stream);
clada_status clada_static_mask_topk(clada_ctx *ctx, const float *score, int32_t d_ff, int32_t k,
                                    int32_t *active_idx, int32_t *n_active, void *hip_stream);

/* Packed mask storage (the paper's limitations name the memory that stored masks
 * take; its future work asks for a sparse encoding): a mask over d_ff neurons as
 * ceil(d_ff/32) words, bit j%32 of word j/32 set iff neuron j is kept -- the layout
 * of clada_sparse_ffn_decode's mask_bits, d_ff/8 bytes against 4 bytes per kept
 * neuron for a list.  clada_mask_pack builds the words from an ascending list
 * (active_idx, n_active[0]); clada_mask_unpack rebuilds the ascending list and its
 * count (bits past d_ff are ignored).  Both exact; all arrays device. */
clada_status clada_mask_pack(clada_ctx *ctx, const int32_t *active_idx, const int32_t *n_active,
                             int32_t d_ff, uint32_t *mask_bits, void *hip_stream);
clada_status clada_mask_unpack(clada_ctx *ctx, const uint32_t *mask_bits, int32_t d_ff,
                               int32_t *active_idx, int32_t *n_active, void *hip_stream);

/* Sparse storage of a mask (the same two passages): the ascending positions j_0 < j_1 < ...
 * at which mask_bits differs from ref_bits, a reference mask of the same layer such as
 * its prefix-static mask or the previous token's mask (ref_bits NULL = the all-zero mask:
 * the positions are the kept neurons), written as the gaps g_i = j_i - j_{i-1} - 1
 * (j_{-1} = -1), each gap a little-endian base-128 number: 7 value bits per byte, low
 * group first, high bit set on every byte but the last.  About one byte per neuron that
 * changed, against d_ff/8 bytes for the bit mask (which no code beats for an unrelated
 * mask at ~50 % sparsity).  Masks are ceil(d_ff/32) words as above; bits past d_ff are
 * ignored on input and zero on output.
 *   clada_mask_sparse_encode: stream [stream_capacity] bytes; n_out [2] = {bytes written,
 *     positions coded}; if the stream does not fit the capacity, n_out[0] = -1 and the
 *     stream's contents are unspecified (n_out[1] is still the number of positions).
 *     clada_mask_sparse_max_bytes(d_ff) is a capacity that always fits.
 *   clada_mask_sparse_decode: mask_bits = ref_bits with the coded positions flipped
 *     (mask_bits may be the same array as ref_bits).  n_bytes [1] is read on the device and
 *     clamped to [0, stream_capacity]; positions >= d_ff and bytes after the last complete
 *     number are ignored, so a damaged stream cannot write out of bounds.
 * Both exact; all arrays device. */
size_t clada_mask_sparse_max_bytes(int32_t d_ff);
clada_status clada_mask_sparse_encode(clada_ctx *ctx, const uint32_t *mask_bits, const uint32_t *ref_bits,
                                      int32_t d_ff, uint8_t *stream, int32_t stream_capacity,
                                      int32_t *n_out, void *hip_stream);
clada_status clada_mask_sparse_decode(clada_ctx *ctx, const uint8_t *stream, const int32_t *n_bytes,
                                      int32_t stream_capacity, const uint32_t *ref_bits, int32_t d_ff,
                                      uint32_t *mask_bits, void *hip_stream);
/* The same for n_masks masks in one launch (1 <= n_masks <= 65535; one workgroup per mask), e.g. the
 * B masks of a layer against its prefix-static mask, or every token's mask against the previous
 * token's: mask m = mask_bits + m * ceil(d_ff/32) words; its reference = ref_bits + m * ref_stride_words
 * (0: one reference for all masks; ref_bits NULL: none); its stream = stream + m * stream_capacity;
 * n_out [n_masks][2]; the decoder reads the byte count of stream m at n_bytes[m * n_bytes_stride]
 * (2 reads the encoder's n_out in place). */
clada_status clada_mask_sparse_encode_batch(clada_ctx *ctx, const uint32_t *mask_bits, const uint32_t *ref_bits,
                                            int64_t ref_stride_words, int32_t d_ff, int32_t n_masks,
                                            uint8_t *stream, int32_t stream_capacity, int32_t *n_out,
                                            void *hip_stream);
clada_status clada_mask_sparse_decode_batch(clada_ctx *ctx, const uint8_t *stream, const int32_t *n_bytes,
                                            int64_t n_bytes_stride, int32_t stream_capacity,
                                            const uint32_t *ref_bits, int64_t ref_stride_words, int32_t d_ff,
                                            int32_t n_masks, uint32_t *mask_bits, void *hip_stream);

/* Sparse SwiGLU FFN over a given neuron list (the sparse forward pass of the
 * algorithm "CLADA Inference" with a mask that does not depend on the token):
 *   y_b = sum_{j in active_idx[0..n_active[0])} SiLU(W_gate[j,:] . x_b) (W_up[j,:] . x_b) W_down[j,:]
 * for every token b of x [B][d].  Only the listed neurons' rows of the three
 * matrices are read.  active_idx ascending int32 in [0,d_ff), n_active [1] int32,
 * both device (e.g. straight from the two calls above, or from
 * clada_sparse_ffn_decode).  Bit-reproducible from run to run. */
clada_status clada_static_ffn_decode(clada_ctx *ctx, const clada_layer *layer, const void *x,
                                     int32_t B, const int32_t *active_idx, const int32_t *n_active,
                                     void *y, void *hip_stream);

/* One decode step as a replayable HIP graph (the algorithm "CLADA Inference", generation
 * phase, is the same short sequence of calls for every token: signals, thresholds, one
 * sparse FFN per layer; captured once, a replay costs one launch instead of 2 L + 2).
 * Between clada_graph_begin and clada_graph_end every call of this library on `hip_stream`
 * (which must not be the default stream) is recorded instead of run; other work the caller
 * enqueues on that stream is recorded too.  The graph holds the pointers the calls were
 * given: replays read and write those same buffers, so the caller refreshes the inputs in
 * place.  Run the same calls once eagerly before capturing (first calls set kernel
 * attributes, which a capture must not contain); options that record events
 * ("diag.kernel_events") must be off.  clada_graph_launch enqueues one replay on
 * `hip_stream`.  The context must outlive the graph; one capture at a time per context. */
typedef struct clada_graph clada_graph;
clada_status clada_graph_begin(clada_ctx *ctx, void *hip_stream);
clada_status clada_graph_end(clada_ctx *ctx, void *hip_stream, clada_graph **out);
clada_status clada_graph_launch(clada_ctx *ctx, clada_graph *graph, void *hip_stream);
void clada_graph_destroy(clada_graph *graph);

/* Measurement helpers (no part of the method).  clada_diag_stream_read reads
 * `bytes` (a multiple of 8192) of device memory once, in the decode kernels'
 * access pattern (each wave streams whole 8 KiB rows with non-temporal 16-byte
 * loads; blocks_per_cu in [1,4] workgroups of 8 waves per compute unit) and
 * discards them: the practical HBM read ceiling.  clada_diag_copy copies `bytes`
 * (a multiple of 16) from src to dst: the known-size transfer the profiler's
 * fetch/write counters are scaled by.  Pointers must be 16-byte aligned. */
/* With option "diag.kernel_events" = 1 a decode call attaches HIP events to its
 * kernels on the call's own stream.  This call waits for the last decode call of
 * the context to finish and returns, in microseconds, the main kernel's own
 * start-to-stop time (main_us) and the final-reduction kernel's (finalize_us; 0
 * for the batched path, whose kernels are timed as one span).  Host pointers. */
clada_status clada_diag_kernel_times(clada_ctx *ctx, float *main_us, float *finalize_us);
clada_status clada_diag_stream_read(clada_ctx *ctx, const void *src, size_t bytes,
                                    int32_t blocks_per_cu, void *hip_stream);
clada_status clada_diag_copy(clada_ctx *ctx, const void *src, void *dst, size_t bytes,
                             void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CLADA_H */
