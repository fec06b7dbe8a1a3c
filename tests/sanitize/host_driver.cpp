// Drives the host-side logic of the library (descriptor checks, workspace queries, launch planning, job-table
// validation, the layer-removal fixed point, SetCoeff) with no GPU: every call below returns before anything is
// enqueued.  Built with the host pass under -fsanitize=address,undefined by tests/test_sanitizers.py, which expects
// "host sanitize ok" and no sanitizer report.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "prunetrain.h"

#define EXPECT(call, want)                                                       \
    do {                                                                         \
        const int32_t rc_ = (call);                                              \
        if (rc_ != (want)) {                                                     \
            std::printf("%s -> %d, expected %d\n", #call, (int)rc_, (int)(want)); \
            return 1;                                                            \
        }                                                                        \
    } while (0)

static pt_conv_desc desc(int N, int H, int W, int C, int K, int R, int st, int pad, int pitch8) {
    pt_conv_desc d;
    std::memset(&d, 0, sizeof d);
    d.struct_size = sizeof d;
    d.N = N; d.H = H; d.W = W; d.C = C; d.K = K; d.R = d.S = R;
    d.stride_h = d.stride_w = st; d.pad_h = d.pad_w = pad;
    d.P = (H + 2 * pad - R) / st + 1; d.Q = (W + 2 * pad - R) / st + 1;
    d.x_cpitch = pitch8 ? (C + 7) / 8 * 8 : C; d.y_cpitch = pitch8 ? (K + 7) / 8 * 8 : K; d.w_cpitch = d.x_cpitch;
    return d;
}

int main() {
    if (pt_version() < 100) return 1;
    // descriptor checks and workspace queries over a spread of shapes (every planning branch, no device work)
    const int shapes[][8] = {{64, 56, 56, 64, 64, 3, 1, 1}, {64, 14, 14, 256, 256, 3, 1, 1}, {64, 7, 7, 2048, 512, 1, 1, 0},
                             {64, 224, 224, 3, 64, 7, 2, 3}, {64, 28, 28, 203, 171, 3, 2, 1}, {2, 9, 9, 19, 131, 3, 2, 1},
                             {1, 1, 1, 8, 8, 1, 1, 0}, {5, 128, 130, 64, 64, 1, 1, 0}, {64, 56, 56, 26, 40, 3, 1, 1}};
    for (const auto& s : shapes)
        for (int p8 = 0; p8 < 2; ++p8) {
            pt_conv_desc d = desc(s[0], s[1], s[2], s[3], s[4], s[5], s[6], s[7], p8);
            size_t b = 0;
            int32_t np = 0;
            EXPECT(pt_conv_fwd_workspace_bytes(&d, &b), PT_OK);
            EXPECT(pt_conv_bwd_data_workspace_bytes(&d, &b), PT_OK);
            EXPECT(pt_conv_bwd_weight_workspace_bytes(&d, &b), PT_OK);
            EXPECT(pt_conv_bwd_weight_lasso_workspace_bytes(&d, &b), PT_OK);
            EXPECT(pt_conv_fwd_stats_workspace_bytes(&d, &b, &np), PT_OK);
            pt_wgrad_plan_info info;
            EXPECT(pt_conv_bwd_weight_plan(&d, p8, &info), PT_OK);
            if (info.splits < 1 || info.tiles < 1) return 1;
            EXPECT(pt_group_norms_workspace_bytes(d.K, d.R * d.S, d.C, &b), PT_OK);
            EXPECT(pt_bn_workspace_bytes((int64_t)d.N * d.P * d.Q, d.K, &b), PT_OK);
            // argument errors are found before anything is enqueued
            EXPECT(pt_conv_fwd(&d, nullptr, nullptr, nullptr, nullptr, 0, nullptr), PT_ERR_NULL);
            EXPECT(pt_conv_bwd_data_crsk(&d, nullptr, nullptr, nullptr, nullptr), PT_ERR_NULL);
            EXPECT(pt_conv_bwd_weight(&d, nullptr, nullptr, nullptr, nullptr, 0, nullptr), PT_ERR_NULL);
            pt_conv_desc bad = d;
            bad.P += 1;
            EXPECT(pt_conv_fwd_workspace_bytes(&bad, &b), PT_ERR_SHAPE);
            bad = d;
            bad.flags = 0x80u;
            EXPECT(pt_conv_bwd_weight_workspace_bytes(&bad, &b), PT_ERR_UNSUPPORTED);
        }
    // multi-layer calls: empty lists and missing pointers
    EXPECT(pt_group_norms_batched(nullptr, 0, nullptr, 0, nullptr), PT_OK);
    pt_layer_weights lw;
    std::memset(&lw, 0, sizeof lw);
    lw.K = 4; lw.RS = 1; lw.C = 8; lw.w_cpitch = 8;
    size_t b = 0;
    EXPECT(pt_group_norms_batched_workspace_bytes(&lw, 1, &b), PT_OK);
    EXPECT(pt_group_norms_batched(&lw, 1, nullptr, 0, nullptr), PT_ERR_NULL);
    pt_layer_detect ld;
    std::memset(&ld, 0, sizeof ld);
    ld.K = 4; ld.RS = 1; ld.C = 8; ld.w_cpitch = 8;
    EXPECT(pt_group_norms_detect_batched_workspace_bytes(&ld, 1, &b), PT_OK);
    EXPECT(pt_group_norms_detect_batched(&ld, 1, 1e-4f, nullptr, 0, nullptr), PT_ERR_NULL);
    EXPECT(pt_group_norms_static(nullptr, 4, 1, 8, 8, nullptr, nullptr, nullptr, nullptr), PT_ERR_NULL);
    EXPECT(pt_group_lasso_grad_batched(nullptr, 0, 1e-3f, nullptr), PT_OK);
    EXPECT(pt_zero_groups_batched(nullptr, 0, 1e-4f, nullptr), PT_OK);
    EXPECT(pt_reconcile_plan_batched(nullptr, 0, nullptr), PT_OK);
    EXPECT(pt_compact_weights_batched(nullptr, 0, nullptr), PT_OK);
    EXPECT(pt_compact_vector_batched(nullptr, 0, nullptr), PT_OK);
    EXPECT(pt_compact_nhwc_batched(nullptr, 0, nullptr), PT_OK);
    EXPECT(pt_weights_to_crsk_batched(nullptr, 0, nullptr), PT_OK);
    // SetCoeff (host arithmetic)
    double lam = 0.0;
    EXPECT(pt_lasso_set_coeff(2.0, 8.0, 0.2, &lam), PT_OK);
    if (!(lam > 0.0624 && lam < 0.0626)) return 1;
    EXPECT(pt_lasso_set_coeff(2.0, 8.0, 1.5, &lam), PT_ERR_SHAPE);
    // layer removal: two blocks on one residual stream; block 0's inner edge has no survivors
    const int32_t p_stream[] = {1, 3}, c_stream[] = {0, 2}, p_in0[] = {0}, c_in0[] = {1}, p_in1[] = {2}, c_in1[] = {3};
    std::vector<pt_removal_edge> edges = {
        {p_stream, c_stream, 2, 2, 16, PT_EDGE_FED_OUTSIDE | PT_EDGE_READ_OUTSIDE},
        {p_in0, c_in0, 1, 1, 0, 0},
        {p_in1, c_in1, 1, 1, 5, 0},
    };
    std::vector<uint8_t> removed(4, 7), dead(3, 7);
    EXPECT(pt_plan_layer_removal(edges.data(), 3, 4, removed.data(), dead.data()), PT_OK);
    if (!(removed[0] == 1 && removed[1] == 1 && removed[2] == 0 && removed[3] == 0 && dead[0] == 0 && dead[1] == 1 && dead[2] == 0)) {
        std::printf("removal plan differs\n");
        return 1;
    }
    edges[0].n_keep = 0;  // the stream itself dies: the network is cut
    EXPECT(pt_plan_layer_removal(edges.data(), 3, 4, removed.data(), dead.data()), PT_ERR_EMPTY);
    std::printf("host sanitize ok\n");
    return 0;
}
