// Context management, status strings and shared argument validation of libclada.
#include <stdarg.h>
#include <stdlib.h>

#include <new>

#include "clada_internal.h"

static thread_local char g_err_no_ctx[256] = "";

clada_status clada_fail(clada_ctx *ctx, clada_status s, const char *fmt, ...)
{
    char *dst = ctx ? ctx->err : g_err_no_ctx;
    size_t cap = ctx ? sizeof(ctx->err) : sizeof(g_err_no_ctx);
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, cap, fmt, ap);
    va_end(ap);
    return s;
}

clada_status clada_check_layer(clada_ctx *ctx, const clada_layer *layer)
{
    if (!layer) return clada_fail(ctx, CLADA_ERR_NULL, "layer is NULL");
    if (layer->kind != CLADA_FFN_SWIGLU && layer->kind != CLADA_FFN_RELU && layer->kind != CLADA_FFN_GEGLU)
        return clada_fail(ctx, CLADA_ERR_VALUE, "unknown FFN kind %d", (int)layer->kind);
    if (!layer->w_gate || !layer->w_down || (layer->kind != CLADA_FFN_RELU && !layer->w_up))
        return clada_fail(ctx, CLADA_ERR_NULL, "a weight pointer is NULL");
    if (layer->dtype != CLADA_F32 && layer->dtype != CLADA_BF16)
        return clada_fail(ctx, CLADA_ERR_DTYPE, "unknown dtype %d", (int)layer->dtype);
    if (layer->d < 1 || layer->d > CLADA_MAX_D)
        return clada_fail(ctx, CLADA_ERR_SHAPE, "d=%d outside [1,%d]", layer->d, CLADA_MAX_D);
    if (layer->d_ff < 1 || layer->d_ff > CLADA_MAX_DFF)
        return clada_fail(ctx, CLADA_ERR_SHAPE, "d_ff=%d outside [1,%d]", layer->d_ff, CLADA_MAX_DFF);
    const size_t rowbytes = (size_t)layer->d * dtype_size(layer->dtype);
    if (rowbytes % 16 != 0)
        return clada_fail(ctx, CLADA_ERR_SHAPE, "row of %zu bytes is not a multiple of 16", rowbytes);
    if (rowbytes > 16384)
        return clada_fail(ctx, CLADA_ERR_SHAPE, "row of %zu bytes exceeds 16384", rowbytes);
    if (!aligned16(layer->w_gate) || !aligned16(layer->w_down) ||
        (layer->kind != CLADA_FFN_RELU && !aligned16(layer->w_up)))
        return clada_fail(ctx, CLADA_ERR_ALIGN, "weight pointers must be 16-byte aligned");
    if (layer->kind == CLADA_FFN_RELU && ((((uintptr_t)layer->b_in) & 3u) || !aligned16(layer->b_out)))
        return clada_fail(ctx, CLADA_ERR_ALIGN, "b_in must be 4-byte and b_out 16-byte aligned");
    return CLADA_OK;
}

clada_status clada_require_swiglu(clada_ctx *ctx, const clada_layer *layer, const char *call)
{
    if (layer->kind == CLADA_FFN_RELU)
        return clada_fail(ctx, CLADA_ERR_VALUE, "%s supports the gated FFN families only", call);
    return CLADA_OK;
}

extern "C" {

clada_status clada_create(clada_ctx **out, int device_id, size_t workspace_bytes)
{
    if (!out) return clada_fail(nullptr, CLADA_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (device_id < 0) return clada_fail(nullptr, CLADA_ERR_VALUE, "device_id=%d", device_id);
    clada_ctx *ctx = new (std::nothrow) clada_ctx();
    if (!ctx) return clada_fail(nullptr, CLADA_ERR_HIP, "host allocation failed");
    ctx->device = device_id;
    ctx->num_cu = 0;
    ctx->ws_bytes = 0;
    ctx->ws = nullptr;
    ctx->opt_decode_wgs_per_cu = 1;
    ctx->opt_decode_b1 = 1;
    ctx->opt_decode_batched = 1;
    ctx->opt_decode_own_first = 0;
    ctx->opt_decode_stack = 3;
    ctx->opt_decode_lane_occ2 = 1;
    ctx->opt_decode_spin_limit = 1 << 12;
    ctx->n_occ = 0;
    ctx->opt_prefix_tile = 0;
    ctx->capturing = 0;
    ctx->opt_diag_events = 0;
    ctx->ev[0] = ctx->ev[1] = ctx->ev[2] = ctx->ev[3] = nullptr;
    for (int i = 0; i < 3; ++i) ctx->lane_stream[i] = nullptr;
    for (int i = 0; i < 4; ++i) ctx->ev_lane[i] = nullptr;
    ctx->err[0] = 0;
    if (workspace_bytes > 0) {
        hipError_t e = hipSetDevice(device_id);
        hipDeviceProp_t prop;
        if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device_id);
        const size_t bytes = align_up(workspace_bytes, 256) + CLADA_WS_HEADER;
        if (e == hipSuccess) e = hipMalloc((void **)&ctx->ws, bytes);
        if (e == hipSuccess) e = hipMemset(ctx->ws, 0, CLADA_WS_HEADER);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) {
            clada_fail(nullptr, CLADA_ERR_HIP, "clada_create: %s", hipGetErrorString(e));
            if (ctx->ws) (void)hipFree(ctx->ws);
            delete ctx;
            return CLADA_ERR_HIP;
        }
        ctx->num_cu = prop.multiProcessorCount;
        ctx->ws_bytes = bytes;
    }
    *out = ctx;
    return CLADA_OK;
}

void clada_destroy(clada_ctx *ctx)
{
    if (!ctx) return;
    for (int i = 0; i < 4; ++i)
        if (ctx->ev[i]) (void)hipEventDestroy(ctx->ev[i]);
    for (int i = 0; i < 4; ++i)
        if (ctx->ev_lane[i]) (void)hipEventDestroy(ctx->ev_lane[i]);
    for (int i = 0; i < 3; ++i)
        if (ctx->lane_stream[i]) (void)hipStreamDestroy(ctx->lane_stream[i]);
    if (ctx->ws) (void)hipFree(ctx->ws);
    delete ctx;
}

const char *clada_status_str(int32_t s)
{
    switch (s) {
    case CLADA_OK: return "CLADA_OK";
    case CLADA_ERR_NULL: return "CLADA_ERR_NULL";
    case CLADA_ERR_SHAPE: return "CLADA_ERR_SHAPE";
    case CLADA_ERR_DTYPE: return "CLADA_ERR_DTYPE";
    case CLADA_ERR_ALIGN: return "CLADA_ERR_ALIGN";
    case CLADA_ERR_WORKSPACE: return "CLADA_ERR_WORKSPACE";
    case CLADA_ERR_VALUE: return "CLADA_ERR_VALUE";
    case CLADA_ERR_HIP: return "CLADA_ERR_HIP";
    }
    return "CLADA_ERR_UNKNOWN";
}

const char *clada_last_error(const clada_ctx *ctx) { return ctx ? ctx->err : g_err_no_ctx; }

clada_status clada_set_option(clada_ctx *ctx, const char *name, int32_t value)
{
    if (!ctx || !name) return clada_fail(ctx, CLADA_ERR_NULL, "ctx or name is NULL");
    if (!strcmp(name, "decode.wgs_per_cu")) {
        if (value < 1 || value > 2) return clada_fail(ctx, CLADA_ERR_VALUE, "decode.wgs_per_cu=%d outside [1,2]", value);
        ctx->opt_decode_wgs_per_cu = value;
        return CLADA_OK;
    }
    if (!strcmp(name, "decode.b1")) {
        if (value < 0 || value > 3) return clada_fail(ctx, CLADA_ERR_VALUE, "decode.b1=%d outside [0,3]", value);
        ctx->opt_decode_b1 = value;
        return CLADA_OK;
    }
    if (!strcmp(name, "decode.batched")) {
        if (value < 0 || value > 1) return clada_fail(ctx, CLADA_ERR_VALUE, "decode.batched=%d outside [0,1]", value);
        ctx->opt_decode_batched = value;
        return CLADA_OK;
    }
    if (!strcmp(name, "decode.lane_occ2")) {
        if (value < 0 || value > 1) return clada_fail(ctx, CLADA_ERR_VALUE, "decode.lane_occ2=%d outside [0,1]", value);
        ctx->opt_decode_lane_occ2 = value;
        return CLADA_OK;
    }
    if (!strcmp(name, "decode.stack")) {
        if (value < 0 || value > 3) return clada_fail(ctx, CLADA_ERR_VALUE, "decode.stack=%d outside [0,3]", value);
        ctx->opt_decode_stack = value;
        return CLADA_OK;
    }
    if (!strcmp(name, "decode.own_first")) {
        if (value < 0 || value > 14) return clada_fail(ctx, CLADA_ERR_VALUE, "decode.own_first=%d outside [0,14]", value);
        ctx->opt_decode_own_first = value;
        return CLADA_OK;
    }
    if (!strcmp(name, "decode.spin_limit")) {
        if (value < 0) return clada_fail(ctx, CLADA_ERR_VALUE, "decode.spin_limit=%d is negative", value);
        ctx->opt_decode_spin_limit = value;
        return CLADA_OK;
    }
    if (!strcmp(name, "prefix.tile")) {
        if (value < 0 || value > 2) return clada_fail(ctx, CLADA_ERR_VALUE, "prefix.tile=%d outside [0,2]", value);
        ctx->opt_prefix_tile = value;
        return CLADA_OK;
    }
    if (!strcmp(name, "diag.kernel_events")) {
        if (value < 0 || value > 1) return clada_fail(ctx, CLADA_ERR_VALUE, "diag.kernel_events=%d outside [0,1]", value);
        if (value && !ctx->ws) return clada_fail(ctx, CLADA_ERR_WORKSPACE, "diag.kernel_events needs a context with a workspace");
        for (int i = 0; value && i < 4; ++i)
            if (!ctx->ev[i]) CLADA_CHECK_HIP(ctx, hipEventCreate(&ctx->ev[i]));
        ctx->opt_diag_events = value;
        return CLADA_OK;
    }
    return clada_fail(ctx, CLADA_ERR_VALUE, "unknown option '%s'", name);
}

clada_status clada_device_fault(clada_ctx *ctx, int32_t *fault_out)
{
    if (!ctx || !fault_out) return clada_fail(ctx, CLADA_ERR_NULL, "ctx or fault_out is NULL");
    if (!ctx->ws) return clada_fail(ctx, CLADA_ERR_WORKSPACE, "the context has no workspace (no device)");
    CLADA_CHECK_HIP(ctx, hipDeviceSynchronize());
    CLADA_CHECK_HIP(ctx, hipMemcpy(fault_out, ctx->ws + COOP_FAULT, sizeof(int32_t), hipMemcpyDeviceToHost));
    return CLADA_OK;
}

clada_status clada_diag_kernel_times(clada_ctx *ctx, float *main_us, float *finalize_us)
{
    if (!ctx || !main_us || !finalize_us) return clada_fail(ctx, CLADA_ERR_NULL, "ctx or an output is NULL");
    if (!ctx->opt_diag_events) return clada_fail(ctx, CLADA_ERR_VALUE, "diag.kernel_events is off");
    CLADA_CHECK_HIP(ctx, hipEventSynchronize(ctx->ev[3]));
    float a = 0.0f, b = 0.0f;
    CLADA_CHECK_HIP(ctx, hipEventElapsedTime(&a, ctx->ev[0], ctx->ev[1]));
    CLADA_CHECK_HIP(ctx, hipEventElapsedTime(&b, ctx->ev[2], ctx->ev[3]));
    *main_us = a * 1e3f;
    *finalize_us = b * 1e3f;
    return CLADA_OK;
}

size_t clada_workspace_bytes(int32_t d, int32_t d_ff, int32_t B, int32_t T, int32_t V)
{
    size_t need = 0, n;
    if (d > 0 && d_ff > 0 && B > 0 && (n = clada_ws_decode(d, d_ff, B)) > need) need = n;
    if (B > 0 && V > 0 && (n = clada_ws_signals(B, V)) > need) need = n;
    if (d > 0 && d_ff > 0 && T > 0 && (n = clada_ws_prefix(d, d_ff, T, true)) > need) need = n;
    if (T > 0 && (n = clada_ws_calibrate()) > need) need = n;
    if (d > 0 && d_ff > 0 && T > 0 && (n = clada_ws_cett(d, d_ff, T)) > need) need = n;
    return need + 256;
}

// ---- one decode step as a HIP graph: thin wrappers over stream capture, so that callers without a
// framework's capture facility can replay the per-token call sequence.
struct clada_graph {
    hipGraph_t graph;
    hipGraphExec_t exec;
};

clada_status clada_graph_begin(clada_ctx *ctx, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    if (!hip_stream) return clada_fail(ctx, CLADA_ERR_VALUE, "the default stream cannot be captured");
    if (!ctx->ws) return clada_fail(ctx, CLADA_ERR_WORKSPACE, "the context has no workspace (no device)");
    if (ctx->opt_diag_events) return clada_fail(ctx, CLADA_ERR_VALUE, "switch diag.kernel_events off before capturing");
    if (ctx->capturing) return clada_fail(ctx, CLADA_ERR_VALUE, "a capture is already open on this context");
    CLADA_CHECK_HIP(ctx, hipStreamBeginCapture((hipStream_t)hip_stream, hipStreamCaptureModeRelaxed));
    ctx->capturing = 1;
    return CLADA_OK;
}

clada_status clada_graph_end(clada_ctx *ctx, void *hip_stream, clada_graph **out)
{
    if (!ctx) return CLADA_ERR_NULL;
    if (!out) return clada_fail(ctx, CLADA_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (!ctx->capturing) return clada_fail(ctx, CLADA_ERR_VALUE, "no capture is open on this context");
    ctx->capturing = 0;
    hipGraph_t g = nullptr;
    CLADA_CHECK_HIP(ctx, hipStreamEndCapture((hipStream_t)hip_stream, &g));
    if (!g) return clada_fail(ctx, CLADA_ERR_HIP, "the capture produced no graph");
    hipGraphExec_t ex = nullptr;
    hipError_t e = hipGraphInstantiate(&ex, g, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        (void)hipGraphDestroy(g);
        CLADA_CHECK_HIP(ctx, e);
    }
    clada_graph *r = new (std::nothrow) clada_graph{g, ex};
    if (!r) {
        (void)hipGraphExecDestroy(ex);
        (void)hipGraphDestroy(g);
        return clada_fail(ctx, CLADA_ERR_HIP, "out of host memory");
    }
    *out = r;
    return CLADA_OK;
}

clada_status clada_graph_launch(clada_ctx *ctx, clada_graph *graph, void *hip_stream)
{
    if (!ctx) return CLADA_ERR_NULL;
    if (!graph) return clada_fail(ctx, CLADA_ERR_NULL, "graph is NULL");
    CLADA_CHECK_HIP(ctx, hipGraphLaunch(graph->exec, (hipStream_t)hip_stream));
    return CLADA_OK;
}

void clada_graph_destroy(clada_graph *graph)
{
    if (!graph) return;
    (void)hipGraphExecDestroy(graph->exec);
    (void)hipGraphDestroy(graph->graph);
    delete graph;
}

}  // extern "C"
