// Walks the host side of the C ABI (argument validation, options, error text, context life cycle) on a
// context without a device, in a build whose host code is instrumented with -fsanitize=address,undefined
// (tests/test_sanitizers.py).  No kernel is launched.  Test infrastructure only.
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "clada.h"

static int fails = 0;
#define EXPECT(call, want) do { const clada_status s_ = (call); if (s_ != (want)) { std::printf("%s -> %d, want %d\n", #call, (int)s_, (int)(want)); ++fails; } } while (0)

int main()
{
    clada_ctx *ctx = nullptr;
    EXPECT(clada_create(nullptr, 0, 0), CLADA_ERR_NULL);
    EXPECT(clada_create(&ctx, 0, 0), CLADA_OK);                 // no workspace: touches no GPU
    alignas(256) static char buf[4096];
    void *p = buf;
    clada_layer ok;
    std::memset(&ok, 0, sizeof(ok));
    ok.w_gate = ok.w_up = ok.w_down = p; ok.d = 64; ok.d_ff = 32; ok.dtype = CLADA_BF16; ok.kind = CLADA_FFN_SWIGLU;
    clada_layer bad = ok;
    float tau = 0.1f;
    // layer descriptors
    bad.d = 0;            EXPECT(clada_dense_ffn_decode(ctx, &bad, p, 1, p, nullptr), CLADA_ERR_SHAPE);
    bad = ok; bad.d = 12; EXPECT(clada_dense_ffn_decode(ctx, &bad, p, 1, p, nullptr), CLADA_ERR_SHAPE);      // row not a multiple of 16 bytes
    bad = ok; bad.dtype = 9; EXPECT(clada_dense_ffn_decode(ctx, &bad, p, 1, p, nullptr), CLADA_ERR_DTYPE);
    bad = ok; bad.kind = 7; EXPECT(clada_dense_ffn_decode(ctx, &bad, p, 1, p, nullptr), CLADA_ERR_VALUE);
    bad = ok; bad.w_up = nullptr; EXPECT(clada_dense_ffn_decode(ctx, &bad, p, 1, p, nullptr), CLADA_ERR_NULL);
    bad = ok; bad.w_gate = buf + 4; EXPECT(clada_dense_ffn_decode(ctx, &bad, p, 1, p, nullptr), CLADA_ERR_ALIGN);
    bad = ok; bad.kind = CLADA_FFN_RELU; bad.w_up = nullptr; bad.b_in = (const float *)(buf + 2);
    EXPECT(clada_dense_ffn_decode(ctx, &bad, p, 1, p, nullptr), CLADA_ERR_ALIGN);
    bad = ok; bad.kind = CLADA_FFN_GEGLU; EXPECT(clada_dense_ffn_decode(ctx, &bad, p, 1, p, nullptr), CLADA_ERR_WORKSPACE);
    // every compute entry point: valid arguments reach the workspace check, invalid ones stop earlier
    EXPECT(clada_sparse_ffn_decode(ctx, &ok, p, 1, &tau, p, nullptr, nullptr, nullptr, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_sparse_ffn_decode(ctx, &ok, p, 0, &tau, p, nullptr, nullptr, nullptr, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_sparse_ffn_decode(ctx, &ok, p, 1, nullptr, p, nullptr, nullptr, nullptr, nullptr), CLADA_ERR_NULL);
    EXPECT(clada_sparse_ffn_decode(ctx, nullptr, p, 1, &tau, p, nullptr, nullptr, nullptr, nullptr), CLADA_ERR_NULL);
    EXPECT(clada_static_ffn_decode(ctx, &ok, p, 1, (const int32_t *)p, (const int32_t *)p, p, nullptr), CLADA_ERR_WORKSPACE);
    clada_prefix_out out;
    std::memset(&out, 0, sizeof(out));
    EXPECT(clada_prefix_stats(ctx, &ok, p, 4, nullptr, &out, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_prefix_stats(ctx, &ok, p, 0, nullptr, &out, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_prefix_stats(ctx, &ok, p, 4, nullptr, nullptr, nullptr), CLADA_ERR_NULL);
    EXPECT(clada_threshold_calibrate(ctx, (const float *)p, 10, 0.4f, (float *)p, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_threshold_calibrate(ctx, (const float *)p, 10, 1.0f, (float *)p, nullptr), CLADA_ERR_VALUE);
    EXPECT(clada_threshold_search_cett(ctx, &ok, p, 4, 0.2f, 31, (float *)p, (float *)p, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_threshold_search_cett(ctx, &ok, p, 4, 0.2f, 0, (float *)p, (float *)p, nullptr), CLADA_ERR_VALUE);
    EXPECT(clada_cett_eval(ctx, &bad, p, 4, 0.1f, (float *)p, (float *)p, nullptr), CLADA_ERR_WORKSPACE);
    bad = ok; bad.kind = CLADA_FFN_RELU; bad.w_up = nullptr;      // the non-gated family is accepted by the CETT calls
    EXPECT(clada_cett_eval(ctx, &bad, p, 4, 0.1f, (float *)p, (float *)p, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_threshold_search_cett(ctx, &bad, p, 4, 0.2f, 31, (float *)p, (float *)p, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_cognitive_signals(ctx, p, CLADA_F32, 1, 10, (const int32_t *)p, (float *)p, (float *)p, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_cognitive_signals(ctx, p, 5, 1, 10, (const int32_t *)p, (float *)p, (float *)p, nullptr), CLADA_ERR_DTYPE);
    EXPECT(clada_cognitive_signals(ctx, p, CLADA_F32, 65, 10, (const int32_t *)p, (float *)p, (float *)p, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_threshold(ctx, (const float *)p, (const float *)p, (const float *)p, 1, (const float *)p, (const float *)p, 1, 0.f, 0.f, (float *)p, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_static_mask_threshold(ctx, (const float *)p, 32, (const float *)p, (int32_t *)p, (int32_t *)p, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_static_mask_topk(ctx, (const float *)p, 32, 33, (int32_t *)p, (int32_t *)p, nullptr), CLADA_ERR_VALUE);
    EXPECT(clada_mask_pack(ctx, (const int32_t *)p, (const int32_t *)p, 0, (uint32_t *)p, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_mask_unpack(ctx, (const uint32_t *)p, 32, (int32_t *)p, (int32_t *)p, nullptr), CLADA_ERR_WORKSPACE);
    // fused signals + thresholds, the variant on the static scratch array, sparse mask storage, whole-stack calls
    EXPECT(clada_signals_threshold(ctx, p, CLADA_F32, 1, 10, (const int32_t *)p, (const float *)p, (const float *)p,
                                   (const float *)p, 0, 0.f, 0.f, (float *)p, (float *)p, (float *)p, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_signals_threshold(ctx, p, CLADA_F32, 1, 10, (const int32_t *)p, (const float *)p, (const float *)p,
                                   (const float *)p, 2, 0.f, 0.f, (float *)p, (float *)p, nullptr, nullptr), CLADA_ERR_NULL);
    EXPECT(clada_signals_threshold(ctx, p, CLADA_F32, 1, 10, (const int32_t *)p, (const float *)p, (const float *)p,
                                   (const float *)p, 2, 0.f, 0.f, (float *)p, (float *)p, (float *)p, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_cognitive_signals_static(ctx, p, CLADA_F32, 1, CLADA_STATIC_SIGNALS_MAX_V + 1, (const int32_t *)p,
                                          (float *)p, (float *)p, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_cognitive_signals_static(ctx, p, 5, 1, 10, (const int32_t *)p, (float *)p, (float *)p, nullptr), CLADA_ERR_DTYPE);
    EXPECT(clada_cognitive_signals_static(nullptr, p, CLADA_F32, 1, 10, (const int32_t *)p, (float *)p, (float *)p, nullptr), CLADA_ERR_NULL);
    if (clada_mask_sparse_max_bytes(0) != 0 || clada_mask_sparse_max_bytes(100) != 100 ||
        clada_mask_sparse_max_bytes(262144) != 262144 + 2048 + 16) ++fails;
    EXPECT(clada_mask_sparse_encode(ctx, (const uint32_t *)p, nullptr, 0, (uint8_t *)p, 16, (int32_t *)p, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_mask_sparse_encode(ctx, (const uint32_t *)p, nullptr, 64, (uint8_t *)p, -1, (int32_t *)p, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_mask_sparse_encode(ctx, (const uint32_t *)p, nullptr, 64, nullptr, 16, (int32_t *)p, nullptr), CLADA_ERR_NULL);
    EXPECT(clada_mask_sparse_encode(ctx, (const uint32_t *)p, nullptr, 64, (uint8_t *)p, 16, (int32_t *)p, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_mask_sparse_decode(ctx, (const uint8_t *)p, (const int32_t *)p, 16, nullptr, 1 << 30, (uint32_t *)p, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_mask_sparse_decode(ctx, (const uint8_t *)p, nullptr, 16, nullptr, 64, (uint32_t *)p, nullptr), CLADA_ERR_NULL);
    EXPECT(clada_mask_sparse_decode(ctx, (const uint8_t *)p, (const int32_t *)p, 16, nullptr, 64, (uint32_t *)p, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_mask_sparse_encode_batch(ctx, (const uint32_t *)p, nullptr, 0, 64, 0, (uint8_t *)p, 16, (int32_t *)p, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_mask_sparse_encode_batch(ctx, (const uint32_t *)p, nullptr, -1, 64, 2, (uint8_t *)p, 16, (int32_t *)p, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_mask_sparse_encode_batch(ctx, (const uint32_t *)p, nullptr, 0, 64, 2, (uint8_t *)p, 16, (int32_t *)p, nullptr), CLADA_ERR_WORKSPACE);
    EXPECT(clada_mask_sparse_decode_batch(ctx, (const uint8_t *)p, (const int32_t *)p, 2, 16, nullptr, 0, 64, 70000, (uint32_t *)p, nullptr), CLADA_ERR_SHAPE);
    EXPECT(clada_mask_sparse_decode_batch(ctx, (const uint8_t *)p, (const int32_t *)p, 2, 16, nullptr, 0, 64, 2, (uint32_t *)p, nullptr), CLADA_ERR_WORKSPACE);
    {
        clada_layer two[2] = {ok, ok};
        EXPECT(clada_sparse_ffn_stack_decode(ctx, nullptr, 2, p, 1, (const float *)p, p, nullptr, nullptr), CLADA_ERR_NULL);
        EXPECT(clada_sparse_ffn_stack_decode(ctx, two, 0, p, 1, (const float *)p, p, nullptr, nullptr), CLADA_ERR_SHAPE);
        EXPECT(clada_sparse_ffn_stack_decode(ctx, two, 2, p, 1, nullptr, p, nullptr, nullptr), CLADA_ERR_NULL);
        EXPECT(clada_sparse_ffn_stack_decode(ctx, two, 2, p, 1, (const float *)p, p, nullptr, nullptr), CLADA_ERR_WORKSPACE);
        EXPECT(clada_sparse_ffn_stack_decode(ctx, two, 2, p, 65, (const float *)p, p, nullptr, nullptr), CLADA_ERR_SHAPE);
        EXPECT(clada_sparse_ffn_stack_decode(ctx, two, 2, p, 8, (const float *)p, p, nullptr, nullptr), CLADA_ERR_WORKSPACE);
        EXPECT(clada_dense_ffn_stack_decode(ctx, two, 2, p, 1, p, nullptr), CLADA_ERR_WORKSPACE);
        two[1].d_ff = ok.d_ff * 2;
        EXPECT(clada_dense_ffn_stack_decode(ctx, two, 2, p, 1, p, nullptr), CLADA_ERR_SHAPE);
    }
    // options, error text, fault query, graph helpers
    EXPECT(clada_set_option(ctx, "decode.stack", 1), CLADA_OK);
    EXPECT(clada_set_option(ctx, "decode.stack", 4), CLADA_ERR_VALUE);
    EXPECT(clada_set_option(ctx, "decode.lane_occ2", 0), CLADA_OK);
    EXPECT(clada_set_option(ctx, "decode.lane_occ2", 2), CLADA_ERR_VALUE);
    EXPECT(clada_set_option(ctx, "decode.b1", 3), CLADA_OK);
    EXPECT(clada_set_option(ctx, "decode.b1", 4), CLADA_ERR_VALUE);
    EXPECT(clada_set_option(ctx, "prefix.tile", 2), CLADA_OK);
    EXPECT(clada_set_option(ctx, "no.such.option", 1), CLADA_ERR_VALUE);
    EXPECT(clada_set_option(ctx, nullptr, 1), CLADA_ERR_NULL);
    EXPECT(clada_set_option(ctx, "diag.kernel_events", 1), CLADA_ERR_WORKSPACE);
    if (!std::strstr(clada_last_error(ctx), "diag.kernel_events")) { std::printf("last error: %s\n", clada_last_error(ctx)); ++fails; }
    int32_t fault = 7;
    EXPECT(clada_device_fault(ctx, &fault), CLADA_ERR_WORKSPACE);
    float a = 0, b = 0;
    EXPECT(clada_diag_kernel_times(ctx, &a, &b), CLADA_ERR_VALUE);
    clada_graph *g = nullptr;
    EXPECT(clada_graph_begin(ctx, nullptr), CLADA_ERR_VALUE);
    EXPECT(clada_graph_begin(ctx, p), CLADA_ERR_WORKSPACE);
    EXPECT(clada_graph_end(ctx, p, &g), CLADA_ERR_VALUE);
    EXPECT(clada_graph_launch(ctx, nullptr, nullptr), CLADA_ERR_NULL);
    clada_graph_destroy(nullptr);
    for (int s = -1; s <= 8; ++s) if (!clada_status_str(s)) ++fails;
    if (std::strcmp(clada_status_str(99), "CLADA_ERR_UNKNOWN") != 0) ++fails;
    if (clada_workspace_bytes(4096, 11008, 1, 512, 32000) < (size_t)(64u << 20)) ++fails;
    if (clada_workspace_bytes(0, 0, 0, 0, 0) > 4096) ++fails;
    clada_destroy(ctx);
    clada_destroy(nullptr);
    std::printf("abi sanitizer driver: %d failures\n", fails);
    return fails ? 1 : 0;
}
