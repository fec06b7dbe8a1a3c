/*
 * CPU oracle (fp64, plain loops) for the PruneTrain conv-layer hot path.
 * TEST INFRASTRUCTURE ONLY - see oracle.h.  No code here is shared with, derived
 * from, or called by the HIP library.
 */
#include "oracle.h"

#include <math.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int oracle_conv_shape_ok(const oracle_conv_shape* s) {
    if (!s) return -1;
    if (s->N <= 0 || s->H <= 0 || s->W <= 0 || s->C <= 0 || s->K <= 0 || s->R <= 0 || s->S <= 0) return -2;
    if (s->stride_h <= 0 || s->stride_w <= 0 || s->pad_h < 0 || s->pad_w < 0) return -2;
    if (s->H + 2 * s->pad_h < s->R || s->W + 2 * s->pad_w < s->S) return -2;
    if (s->P != (s->H + 2 * s->pad_h - s->R) / s->stride_h + 1) return -2;
    if (s->Q != (s->W + 2 * s->pad_w - s->S) / s->stride_w + 1) return -2;
    return 0;
}

/* element accessors for the dense layouts */
static inline size_t xi(const oracle_conv_shape* s, int n, int h, int w, int c) {
    return (((size_t)n * s->H + h) * s->W + w) * s->C + c;
}
static inline size_t yi(const oracle_conv_shape* s, int n, int p, int q, int k) {
    return (((size_t)n * s->P + p) * s->Q + q) * s->K + k;
}
static inline size_t wi(const oracle_conv_shape* s, int k, int r, int t, int c) {
    return (((size_t)k * s->R + r) * s->S + t) * s->C + c;
}

/* one output element of the forward map (Sec. 2.1) */
static double fwd_elem(const oracle_conv_shape* s, const double* x, const double* w, int n, int p, int q, int k) {
    double acc = 0.0;
    for (int r = 0; r < s->R; ++r) {
        int h = p * s->stride_h - s->pad_h + r;
        if (h < 0 || h >= s->H) continue;
        for (int t = 0; t < s->S; ++t) {
            int ww = q * s->stride_w - s->pad_w + t;
            if (ww < 0 || ww >= s->W) continue;
            for (int c = 0; c < s->C; ++c) acc += x[xi(s, n, h, ww, c)] * w[wi(s, k, r, t, c)];
        }
    }
    return acc;
}

/* one element of the input gradient: every (p,r) pair with p*st - pad + r == h contributes */
static double bwd_data_elem(const oracle_conv_shape* s, const double* dy, const double* w, int n, int h, int ww,
                            int c) {
    double acc = 0.0;
    for (int r = 0; r < s->R; ++r) {
        int hp = h + s->pad_h - r;
        if (hp < 0 || hp % s->stride_h != 0) continue;
        int p = hp / s->stride_h;
        if (p >= s->P) continue;
        for (int t = 0; t < s->S; ++t) {
            int wq = ww + s->pad_w - t;
            if (wq < 0 || wq % s->stride_w != 0) continue;
            int q = wq / s->stride_w;
            if (q >= s->Q) continue;
            for (int k = 0; k < s->K; ++k) acc += dy[yi(s, n, p, q, k)] * w[wi(s, k, r, t, c)];
        }
    }
    return acc;
}

/* one element of the weight gradient (Eq. 4): plain sum over the mini-batch and all output pixels */
static double bwd_weight_elem(const oracle_conv_shape* s, const double* x, const double* dy, int k, int r, int t,
                              int c) {
    double acc = 0.0;
    for (int n = 0; n < s->N; ++n) {
        for (int p = 0; p < s->P; ++p) {
            int h = p * s->stride_h - s->pad_h + r;
            if (h < 0 || h >= s->H) continue;
            for (int q = 0; q < s->Q; ++q) {
                int ww = q * s->stride_w - s->pad_w + t;
                if (ww < 0 || ww >= s->W) continue;
                acc += dy[yi(s, n, p, q, k)] * x[xi(s, n, h, ww, c)];
            }
        }
    }
    return acc;
}

int oracle_conv_fwd(const oracle_conv_shape* s, const double* x, const double* w, double* y) {
    int rc = oracle_conv_shape_ok(s);
    if (rc) return rc;
    if (!x || !w || !y) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < s->N; ++n)
        for (int p = 0; p < s->P; ++p)
            for (int q = 0; q < s->Q; ++q)
                for (int k = 0; k < s->K; ++k) y[yi(s, n, p, q, k)] = fwd_elem(s, x, w, n, p, q, k);
    return 0;
}

int oracle_conv_bwd_data(const oracle_conv_shape* s, const double* dy, const double* w, double* dx) {
    int rc = oracle_conv_shape_ok(s);
    if (rc) return rc;
    if (!dy || !w || !dx) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < s->N; ++n)
        for (int h = 0; h < s->H; ++h)
            for (int ww = 0; ww < s->W; ++ww)
                for (int c = 0; c < s->C; ++c) dx[xi(s, n, h, ww, c)] = bwd_data_elem(s, dy, w, n, h, ww, c);
    return 0;
}

int oracle_conv_bwd_weight(const oracle_conv_shape* s, const double* x, const double* dy, double* dw) {
    int rc = oracle_conv_shape_ok(s);
    if (rc) return rc;
    if (!x || !dy || !dw) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < s->K; ++k)
        for (int r = 0; r < s->R; ++r)
            for (int t = 0; t < s->S; ++t)
                for (int c = 0; c < s->C; ++c) dw[wi(s, k, r, t, c)] = bwd_weight_elem(s, x, dy, k, r, t, c);
    return 0;
}

int oracle_conv_fwd_at(const oracle_conv_shape* s, const double* x, const double* w, const int64_t* idx,
                       int64_t n_idx, double* out) {
    int rc = oracle_conv_shape_ok(s);
    if (rc) return rc;
    if (!x || !w || !idx || !out) return -1;
    const int64_t total = (int64_t)s->N * s->P * s->Q * s->K;
    for (int64_t i = 0; i < n_idx; ++i)
        if (idx[i] < 0 || idx[i] >= total) return -2;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t f = idx[i];
        int k = (int)(f % s->K); f /= s->K;
        int q = (int)(f % s->Q); f /= s->Q;
        int p = (int)(f % s->P); f /= s->P;
        out[i] = fwd_elem(s, x, w, (int)f, p, q, k);
    }
    return 0;
}

int oracle_conv_bwd_data_at(const oracle_conv_shape* s, const double* dy, const double* w, const int64_t* idx,
                            int64_t n_idx, double* out) {
    int rc = oracle_conv_shape_ok(s);
    if (rc) return rc;
    if (!dy || !w || !idx || !out) return -1;
    const int64_t total = (int64_t)s->N * s->H * s->W * s->C;
    for (int64_t i = 0; i < n_idx; ++i)
        if (idx[i] < 0 || idx[i] >= total) return -2;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t f = idx[i];
        int c = (int)(f % s->C); f /= s->C;
        int ww = (int)(f % s->W); f /= s->W;
        int h = (int)(f % s->H); f /= s->H;
        out[i] = bwd_data_elem(s, dy, w, (int)f, h, ww, c);
    }
    return 0;
}

int oracle_conv_bwd_weight_at(const oracle_conv_shape* s, const double* x, const double* dy, const int64_t* idx,
                              int64_t n_idx, double* out) {
    int rc = oracle_conv_shape_ok(s);
    if (rc) return rc;
    if (!x || !dy || !idx || !out) return -1;
    const int64_t total = (int64_t)s->K * s->R * s->S * s->C;
    for (int64_t i = 0; i < n_idx; ++i)
        if (idx[i] < 0 || idx[i] >= total) return -2;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t f = idx[i];
        int c = (int)(f % s->C); f /= s->C;
        int t = (int)(f % s->S); f /= s->S;
        int r = (int)(f % s->R); f /= s->R;
        out[i] = bwd_weight_elem(s, x, dy, (int)f, r, t, c);
    }
    return 0;
}

int oracle_group_norms(const double* w, int32_t K, int32_t RS, int32_t C, double* out_norm, double* in_norm) {
    if (!w || !out_norm || !in_norm) return -1;
    if (K <= 0 || RS <= 0 || C <= 0) return -2;
    /* output-channel group k: every weight of filter k */
    for (int k = 0; k < K; ++k) {
        double ss = 0.0;
        for (int j = 0; j < RS; ++j)
            for (int c = 0; c < C; ++c) {
                double v = w[((size_t)k * RS + j) * C + c];
                ss += v * v;
            }
        out_norm[k] = sqrt(ss);
    }
    /* input-channel group c: every weight that multiplies input channel c */
    for (int c = 0; c < C; ++c) {
        double ss = 0.0;
        for (int k = 0; k < K; ++k)
            for (int j = 0; j < RS; ++j) {
                double v = w[((size_t)k * RS + j) * C + c];
                ss += v * v;
            }
        in_norm[c] = sqrt(ss);
    }
    return 0;
}

int oracle_group_lasso_grad(const double* w, const double* out_norm, const double* in_norm, double lambda,
                            uint32_t flags, double* dw, int32_t K, int32_t RS, int32_t C) {
    if (!w || !out_norm || !in_norm || !dw) return -1;
    if (K <= 0 || RS <= 0 || C <= 0) return -2;
    const int reg_out = (flags & 1u) != 0, reg_in = (flags & 2u) != 0;
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < RS; ++j)
            for (int c = 0; c < C; ++c) {
                size_t i = ((size_t)k * RS + j) * C + c;
                double g = 0.0;
                if (reg_out && out_norm[k] > 0.0) g += w[i] / out_norm[k];
                if (reg_in && in_norm[c] > 0.0) g += w[i] / in_norm[c];
                dw[i] += lambda * g;
            }
    return 0;
}

int oracle_group_lasso_penalty(const double* out_norm, int32_t K, const double* in_norm, int32_t C, uint32_t flags,
                               double* penalty) {
    if (!penalty || (K > 0 && !out_norm) || (C > 0 && !in_norm)) return -1;
    if (K < 0 || C < 0) return -2;
    double p = 0.0;
    if (flags & 1u)
        for (int k = 0; k < K; ++k) p += out_norm[k];
    if (flags & 2u)
        for (int c = 0; c < C; ++c) p += in_norm[c];
    *penalty += p;
    return 0;
}

int oracle_set_coeff(double loss1, double loss2, double ratio, double* lambda) {
    if (!lambda) return -1;
    if (!(ratio > 0.0 && ratio < 1.0) || !(loss2 > 0.0) || !(loss1 >= 0.0)) return -2;
    *lambda = ratio * loss1 / ((1.0 - ratio) * loss2);
    return 0;
}

int oracle_zero_groups(const double* norms, int32_t n, double thr, uint8_t* zero) {
    if (!norms || !zero) return -1;
    if (n < 0) return -2;
    for (int i = 0; i < n; ++i) zero[i] = (uint8_t)(norms[i] < thr);
    return 0;
}

int oracle_reconcile_edge(const uint8_t* const* producer_zero, int32_t n_prod, const uint8_t* const* consumer_zero,
                          int32_t n_cons, int32_t n, uint8_t* keep) {
    if (!keep || (n_prod > 0 && !producer_zero) || (n_cons > 0 && !consumer_zero)) return -1;
    if (n < 0 || n_prod < 0 || n_cons < 0 || n_prod + n_cons == 0) return -2;
    for (int j = 0; j < n; ++j) {
        int all_zero = 1;
        for (int a = 0; a < n_prod; ++a)
            if (!producer_zero[a][j]) all_zero = 0;
        for (int b = 0; b < n_cons; ++b)
            if (!consumer_zero[b][j]) all_zero = 0;
        keep[j] = (uint8_t)!all_zero;
    }
    return 0;
}

int oracle_compact_plan(const uint8_t* keep, int32_t n, int32_t* idx, int32_t* n_keep) {
    if (!keep || !idx || !n_keep) return -1;
    if (n < 0) return -2;
    int32_t m = 0;
    for (int j = 0; j < n; ++j)
        if (keep[j]) idx[m++] = j;
    *n_keep = m;
    return 0;
}

int oracle_compact_weights(const double* w, int32_t K, int32_t RS, int32_t C, const int32_t* idxK, int32_t Kp,
                           const int32_t* idxC, int32_t Cp, double* w_out) {
    if (!w || !w_out) return -1;
    if (K <= 0 || RS <= 0 || C <= 0 || Kp <= 0 || Cp <= 0) return -2;
    if ((!idxK && Kp != K) || (!idxC && Cp != C)) return -2;
    for (int a = 0; a < Kp; ++a) {
        int k = idxK ? idxK[a] : a;
        if (k < 0 || k >= K) return -2;
        for (int j = 0; j < RS; ++j)
            for (int b = 0; b < Cp; ++b) {
                int c = idxC ? idxC[b] : b;
                if (c < 0 || c >= C) return -2;
                w_out[((size_t)a * RS + j) * Cp + b] = w[((size_t)k * RS + j) * C + c];
            }
    }
    return 0;
}

int oracle_compact_vector(const void* v, int32_t elem_bytes, const int32_t* idx, int32_t n_keep, void* out) {
    if (!v || !idx || !out) return -1;
    if (elem_bytes <= 0 || n_keep < 0) return -2;
    for (int j = 0; j < n_keep; ++j)
        memcpy((char*)out + (size_t)j * elem_bytes, (const char*)v + (size_t)idx[j] * elem_bytes, (size_t)elem_bytes);
    return 0;
}

int oracle_compact_nhwc(const void* x, int64_t pixels, int32_t C, int32_t elem_bytes, const int32_t* idx, int32_t Cp,
                        void* out) {
    if (!x || !idx || !out) return -1;
    if (pixels < 0 || C <= 0 || Cp <= 0 || elem_bytes <= 0) return -2;
    for (int b = 0; b < Cp; ++b)
        if (idx[b] < 0 || idx[b] >= C) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < pixels; ++p)
        for (int b = 0; b < Cp; ++b)
            memcpy((char*)out + ((size_t)p * Cp + b) * elem_bytes,
                   (const char*)x + ((size_t)p * C + idx[b]) * elem_bytes, (size_t)elem_bytes);
    return 0;
}

int oracle_scatter_nhwc(const void* x, int64_t pixels, int32_t Cp, int32_t elem_bytes, const int32_t* idx, int32_t C,
                        void* out) {
    if (!x || !idx || !out) return -1;
    if (pixels < 0 || C <= 0 || Cp <= 0 || Cp > C || elem_bytes <= 0) return -2;
    for (int b = 0; b < Cp; ++b) {
        if (idx[b] < 0 || idx[b] >= C) return -2;
        if (b > 0 && idx[b] <= idx[b - 1]) return -2; /* survivor lists are strictly ascending */
    }
    memset(out, 0, (size_t)pixels * C * elem_bytes);
    for (int64_t p = 0; p < pixels; ++p)
        for (int b = 0; b < Cp; ++b)
            memcpy((char*)out + ((size_t)p * C + idx[b]) * elem_bytes,
                   (const char*)x + ((size_t)p * Cp + b) * elem_bytes, (size_t)elem_bytes);
    return 0;
}

int oracle_group_maxabs(const double* w, int32_t K, int32_t RS, int32_t C, double* out_max, double* in_max) {
    if (!w || !out_max || !in_max) return -1;
    if (K <= 0 || RS <= 0 || C <= 0) return -2;
    for (int k = 0; k < K; ++k) {
        double m = 0.0;
        for (int j = 0; j < RS; ++j)
            for (int c = 0; c < C; ++c) {
                double v = fabs(w[((size_t)k * RS + j) * C + c]);
                if (v > m) m = v;
            }
        out_max[k] = m;
    }
    for (int c = 0; c < C; ++c) {
        double m = 0.0;
        for (int k = 0; k < K; ++k)
            for (int j = 0; j < RS; ++j) {
                double v = fabs(w[((size_t)k * RS + j) * C + c]);
                if (v > m) m = v;
            }
        in_max[c] = m;
    }
    return 0;
}

int oracle_apply_zero(double* w, int32_t K, int32_t RS, int32_t C, const uint8_t* zero_out, const uint8_t* zero_in) {
    if (!w) return -1;
    if (K <= 0 || RS <= 0 || C <= 0) return -2;
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < RS; ++j)
            for (int c = 0; c < C; ++c)
                if ((zero_out && zero_out[k]) || (zero_in && zero_in[c])) w[((size_t)k * RS + j) * C + c] = 0.0;
    return 0;
}

int oracle_sgd_momentum_lasso(double* w, const double* dw, double* mom, const double* out_norm, const double* in_norm,
                              double lambda, double lr, double mu, double wd, uint32_t flags, int32_t K, int32_t RS,
                              int32_t C) {
    if (!w || !dw || !mom || !out_norm || !in_norm) return -1;
    if (K <= 0 || RS <= 0 || C <= 0) return -2;
    const int reg_out = (flags & 1u) != 0, reg_in = (flags & 2u) != 0;
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < RS; ++j)
            for (int c = 0; c < C; ++c) {
                size_t i = ((size_t)k * RS + j) * C + c;
                double g = dw[i] + wd * w[i];
                if (reg_out && out_norm[k] > 0.0) g += lambda * w[i] / out_norm[k];
                if (reg_in && in_norm[c] > 0.0) g += lambda * w[i] / in_norm[c];
                mom[i] = mu * mom[i] + g;
                w[i] -= lr * mom[i];
            }
    return 0;
}

int oracle_bn_fwd(const double* x, int64_t pixels, int32_t C, const double* gamma, const double* beta, double eps,
                  double* y, double* mean, double* invstd) {
    if (!x || !gamma || !beta || !y || !mean || !invstd) return -1;
    if (pixels <= 0 || C <= 0 || !(eps >= 0.0)) return -2;
    for (int c = 0; c < C; ++c) {
        double m = 0.0;
        for (int64_t p = 0; p < pixels; ++p) m += x[(size_t)p * C + c];
        m /= (double)pixels;
        double v = 0.0;
        for (int64_t p = 0; p < pixels; ++p) {
            double d = x[(size_t)p * C + c] - m;
            v += d * d;
        }
        v /= (double)pixels; /* biased variance: the batch statistic used for normalisation */
        mean[c] = m;
        invstd[c] = 1.0 / sqrt(v + eps);
        for (int64_t p = 0; p < pixels; ++p) y[(size_t)p * C + c] = (x[(size_t)p * C + c] - m) * invstd[c] * gamma[c] + beta[c];
    }
    return 0;
}

int oracle_bn_bwd(const double* x, const double* dy, int64_t pixels, int32_t C, const double* gamma, const double* mean,
                  const double* invstd, double* dx, double* dgamma, double* dbeta) {
    if (!x || !dy || !gamma || !mean || !invstd || !dx || !dgamma || !dbeta) return -1;
    if (pixels <= 0 || C <= 0) return -2;
    for (int c = 0; c < C; ++c) {
        double sg = 0.0, sb = 0.0;
        for (int64_t p = 0; p < pixels; ++p) {
            double xh = (x[(size_t)p * C + c] - mean[c]) * invstd[c];
            sg += dy[(size_t)p * C + c] * xh;
            sb += dy[(size_t)p * C + c];
        }
        dgamma[c] = sg;
        dbeta[c] = sb;
        for (int64_t p = 0; p < pixels; ++p) {
            double xh = (x[(size_t)p * C + c] - mean[c]) * invstd[c];
            dx[(size_t)p * C + c] = gamma[c] * invstd[c] * (dy[(size_t)p * C + c] - sb / (double)pixels - xh * sg / (double)pixels);
        }
    }
    return 0;
}
