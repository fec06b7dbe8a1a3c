/* Exercises every function of the CPU oracle on small heap buffers of exactly the documented sizes, so that a
 * build with -fsanitize=address,undefined reports any access outside them (tests/test_sanitizers.py builds and runs
 * it).  Prints "oracle sanitize ok" when every call returned 0. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "oracle.h"

static double* dbuf(size_t n, double seed) {
    double* p = (double*)malloc((n ? n : 1) * sizeof(double));
    for (size_t i = 0; i < n; ++i) p[i] = seed * (double)((i * 2654435761u) % 1000) / 1000.0 - 0.3;
    return p;
}
#define CHECK(call) do { int rc_ = (call); if (rc_ != 0) { printf("%s -> %d\n", #call, rc_); return 1; } } while (0)

static int conv_case(int N, int H, int W, int C, int K, int R, int st, int pad) {
    oracle_conv_shape s = {N, H, W, C, K, R, R, st, st, pad, pad, (H + 2 * pad - R) / st + 1, (W + 2 * pad - R) / st + 1};
    CHECK(oracle_conv_shape_ok(&s));
    const size_t nx = (size_t)N * H * W * C, ny = (size_t)N * s.P * s.Q * K, nw = (size_t)K * R * R * C;
    double *x = dbuf(nx, 1.0), *w = dbuf(nw, 0.5), *dy = dbuf(ny, 0.7), *y = dbuf(ny, 0), *dx = dbuf(nx, 0), *dw = dbuf(nw, 0);
    CHECK(oracle_conv_fwd(&s, x, w, y));
    CHECK(oracle_conv_bwd_data(&s, dy, w, dx));
    CHECK(oracle_conv_bwd_weight(&s, x, dy, dw));
    int64_t iy[3] = {0, (int64_t)ny / 2, (int64_t)ny - 1}, ix[3] = {0, (int64_t)nx / 2, (int64_t)nx - 1},
            iw[3] = {0, (int64_t)nw / 2, (int64_t)nw - 1};
    double out[3];
    CHECK(oracle_conv_fwd_at(&s, x, w, iy, 3, out));
    if (out[2] != y[ny - 1]) { printf("fwd_at mismatch\n"); return 1; }
    CHECK(oracle_conv_bwd_data_at(&s, dy, w, ix, 3, out));
    if (out[0] != dx[0]) { printf("bwd_data_at mismatch\n"); return 1; }
    CHECK(oracle_conv_bwd_weight_at(&s, x, dy, iw, 3, out));
    if (out[1] != dw[nw / 2]) { printf("bwd_weight_at mismatch\n"); return 1; }
    free(x); free(w); free(dy); free(y); free(dx); free(dw);
    return 0;
}

int main(void) {
    if (conv_case(2, 5, 6, 3, 4, 3, 1, 1) || conv_case(1, 7, 7, 2, 3, 3, 2, 1) || conv_case(2, 4, 4, 5, 2, 1, 2, 0) ||
        conv_case(1, 9, 8, 1, 2, 5, 3, 2))
        return 1;
    enum { K = 5, RS = 4, C = 7 };
    double *w = dbuf(K * RS * C, 1.0), *dw = dbuf(K * RS * C, 0.2), *mom = dbuf(K * RS * C, 0.1);
    double *on = dbuf(K, 0), *in = dbuf(C, 0), *om = dbuf(K, 0), *im = dbuf(C, 0), pen = 0.0, lam = 0.0;
    CHECK(oracle_group_norms(w, K, RS, C, on, in));
    CHECK(oracle_group_maxabs(w, K, RS, C, om, im));
    CHECK(oracle_group_lasso_grad(w, on, in, 1e-3, 3u, dw, K, RS, C));
    CHECK(oracle_group_lasso_penalty(on, K, in, C, 3u, &pen));
    CHECK(oracle_set_coeff(2.0, pen, 0.2, &lam));
    CHECK(oracle_sgd_momentum_lasso(w, dw, mom, on, in, lam, 0.1, 0.9, 1e-4, 3u, K, RS, C));
    uint8_t *zo = (uint8_t*)malloc(K), *zi = (uint8_t*)malloc(C), *zi2 = (uint8_t*)malloc(C), *keep = (uint8_t*)malloc(C);
    CHECK(oracle_zero_groups(on, K, 0.5, zo));
    CHECK(oracle_zero_groups(in, C, 0.5, zi));
    memset(zi2, 1, C); zi2[C - 1] = 0;
    CHECK(oracle_apply_zero(w, K, RS, C, zo, zi));
    CHECK(oracle_apply_zero(w, K, RS, C, NULL, NULL));
    const uint8_t* prods[1] = {zi};
    const uint8_t* cons[1] = {zi2};
    CHECK(oracle_reconcile_edge(prods, 1, cons, 1, C, keep));
    CHECK(oracle_reconcile_edge(NULL, 0, cons, 1, C, keep));
    int32_t *idx = (int32_t*)malloc(C * sizeof(int32_t)), nk = 0;
    CHECK(oracle_compact_plan(keep, C, idx, &nk));
    if (nk < 1 || nk > C) { printf("plan count %d\n", nk); return 1; }
    double* wc = dbuf((size_t)K * RS * nk, 0);
    CHECK(oracle_compact_weights(w, K, RS, C, NULL, K, idx, nk, wc));
    float vin[C], *vout = (float*)malloc(nk * sizeof(float));
    for (int i = 0; i < C; ++i) vin[i] = (float)i;
    CHECK(oracle_compact_vector(vin, 4, idx, nk, vout));
    enum { PIX = 6 };
    uint16_t *act = (uint16_t*)malloc(PIX * C * 2), *actc = (uint16_t*)malloc((size_t)PIX * nk * 2), *back = (uint16_t*)malloc(PIX * C * 2);
    for (int i = 0; i < PIX * C; ++i) act[i] = (uint16_t)(i + 1);
    CHECK(oracle_compact_nhwc(act, PIX, C, 2, idx, nk, actc));
    CHECK(oracle_scatter_nhwc(actc, PIX, nk, 2, idx, C, back));
    double *bx = dbuf(PIX * C, 1.0), *bdy = dbuf(PIX * C, 0.4), *g = dbuf(C, 1.0), *b = dbuf(C, 0.5), *by = dbuf(PIX * C, 0),
           *mean = dbuf(C, 0), *istd = dbuf(C, 0), *bdx = dbuf(PIX * C, 0), *dg = dbuf(C, 0), *db = dbuf(C, 0);
    CHECK(oracle_bn_fwd(bx, PIX, C, g, b, 1e-5, by, mean, istd));
    CHECK(oracle_bn_bwd(bx, bdy, PIX, C, g, mean, istd, bdx, dg, db));
    oracle_set_num_threads(2);
    if (oracle_num_threads() < 1) return 1;
    free(w); free(dw); free(mom); free(on); free(in); free(om); free(im); free(zo); free(zi); free(zi2); free(keep);
    free(idx); free(wc); free(vout); free(act); free(actc); free(back);
    free(bx); free(bdy); free(g); free(b); free(by); free(mean); free(istd); free(bdx); free(dg); free(db);
    printf("oracle sanitize ok\n");
    return 0;
}
