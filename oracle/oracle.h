/*
 * CPU oracle for the PruneTrain conv-layer hot path.  TEST INFRASTRUCTURE ONLY:
 * it is called by the tests, by the smoke check and by the benchmark's CPU
 * baseline leg, never by the product path, and it shares no code with the HIP
 * library.
 *
 * Everything is fp64 on host pointers, written as the defining formulas with
 * plain nested loops (no im2col, no GEMM, no blocking).  OpenMP only splits the
 * outermost independent loop.
 *
 * Layouts: activations NHWC  x[N][H][W][C], y[N][P][Q][K];
 *          weights     KRSC  w[K][R][S][C];  all dense (pitch == extent).
 * P = (H + 2*pad_h - R)/stride_h + 1, Q likewise.
 *
 * Every pinned function is checked by tests/test_oracle_*.py against closed
 * forms, adjoint identities, finite differences, library routines and brute
 * force; none is "parity unpinned".
 */
#ifndef PRUNETRAIN_ORACLE_H
#define PRUNETRAIN_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, P, Q;
} oracle_conv_shape;

/* Returns 0 when P,Q agree with the formula above and all extents are > 0. */
int oracle_conv_shape_ok(const oracle_conv_shape* s);

/* Forward convolution (cross-correlation, zero padding; Sec. 2.1, Alg. 1 ForwardProp):
 * y[n,p,q,k] = sum_{r,s,c} x[n, p*st-pad+r, q*st-pad+s, c] * w[k,r,s,c]. */
int oracle_conv_fwd(const oracle_conv_shape* s, const double* x, const double* w, double* y);

/* Gradient w.r.t. the input (adjoint of the forward map in x; Alg. 1 BackProp):
 * dx[n,h,w,c] = sum over (p,q,k,r,s) with p*st-pad+r == h, q*st-pad+s == w of dy[n,p,q,k]*w[k,r,s,c]. */
int oracle_conv_bwd_data(const oracle_conv_shape* s, const double* dy, const double* w, double* dx);

/* Gradient w.r.t. the weights (Eq. 4): dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n,p*st-pad+r,q*st-pad+s,c]. */
int oracle_conv_bwd_weight(const oracle_conv_shape* s, const double* x, const double* dy, double* dw);

/* The same three maps evaluated only at the listed flat output indices
 * (idx[i] indexes y / dx / dw in their dense layouts); out[i] receives the value. */
int oracle_conv_fwd_at(const oracle_conv_shape* s, const double* x, const double* w,
                       const int64_t* idx, int64_t n_idx, double* out);
int oracle_conv_bwd_data_at(const oracle_conv_shape* s, const double* dy, const double* w,
                            const int64_t* idx, int64_t n_idx, double* out);
int oracle_conv_bwd_weight_at(const oracle_conv_shape* s, const double* x, const double* dy,
                              const int64_t* idx, int64_t n_idx, double* out);

/* Channel-group L2 norms of one layer (Eq. 2): out_norm[k] = ||w[k,:,:,:]||_2 (filter k),
 * in_norm[c] = ||w[:,:,:,c]||_2 (all weights that multiply input channel c). RS = R*S. */
int oracle_group_norms(const double* w, int32_t K, int32_t RS, int32_t C, double* out_norm, double* in_norm);

/* Gradient of lambda * (sum_k out_norm[k] + sum_c in_norm[c]) added onto dw (Eq. 1-2):
 * dw[k,rs,c] += lambda * w[k,rs,c] * (a/out_norm[k] + b/in_norm[c]); a = flags bit 0,
 * b = flags bit 1; a term whose norm is 0 contributes 0 (minimum-norm subgradient). */
int oracle_group_lasso_grad(const double* w, const double* out_norm, const double* in_norm, double lambda,
                            uint32_t flags, double* dw, int32_t K, int32_t RS, int32_t C);

/* One layer's share of the regulariser's value (Eq. 1-2; GroupLassoReg of Alg. 1), ADDED onto *penalty:
 * a * sum_k out_norm[k] + b * sum_c in_norm[c], a = flags bit 0, b = flags bit 1 (no size weighting: one
 * global coefficient, Sec. 4.1). */
int oracle_group_lasso_penalty(const double* out_norm, int32_t K, const double* in_norm, int32_t C, uint32_t flags,
                               double* penalty);

/* SetCoeff of Alg. 1: the coefficient for which the regulariser makes up `ratio` of the total loss
 * (penalty-ratio equation of Sec. 4.1): ratio = lambda*loss2 / (loss1 + lambda*loss2), solved for lambda.
 * Needs 0 < ratio < 1, loss2 > 0, loss1 >= 0. */
int oracle_set_coeff(double loss1, double loss2, double ratio, double* lambda);

/* zero[g] = (norms[g] < thr) (Sec. 4.1, threshold zeroing; strict comparison). */
int oracle_zero_groups(const double* norms, int32_t n, double thr, uint8_t* zero);

/* Channel edge reconciliation (Sec. 4.2: adjacent-layer intersection and channel union):
 * channel j is dropped only when it is zero in every producer's output groups AND in every
 * consumer's input groups; keep[j] = !that. */
int oracle_reconcile_edge(const uint8_t* const* producer_zero, int32_t n_prod,
                          const uint8_t* const* consumer_zero, int32_t n_cons, int32_t n, uint8_t* keep);

/* Ascending list of surviving indices; *n_keep = how many. */
int oracle_compact_plan(const uint8_t* keep, int32_t n, int32_t* idx, int32_t* n_keep);

/* w_out[k',rs,c'] = w[idxK[k'],rs,idxC[c']]; a NULL index list is the identity on that axis
 * (then Kp / Cp must equal K / C). */
int oracle_compact_weights(const double* w, int32_t K, int32_t RS, int32_t C, const int32_t* idxK, int32_t Kp,
                           const int32_t* idxC, int32_t Cp, double* w_out);

/* out[j'] = v[idx[j']] for elements of elem_bytes bytes each. */
int oracle_compact_vector(const void* v, int32_t elem_bytes, const int32_t* idx, int32_t n_keep, void* out);

/* out[pix,c'] = x[pix,idx[c']] for elements of elem_bytes bytes each (NHWC activation gather). */
int oracle_compact_nhwc(const void* x, int64_t pixels, int32_t C, int32_t elem_bytes, const int32_t* idx, int32_t Cp,
                        void* out);

/* Threads OpenMP will use for the loops above. */
int oracle_num_threads(void);
void oracle_set_num_threads(int n);

/* Channel scatter (the inverse of the activation gather; the scatter layer of channel gating, Sec. 4.2):
 * out[pix, idx[c']] = x[pix, c'] for c' < Cp, every other channel of out is zero.  idx strictly ascending. */
int oracle_scatter_nhwc(const void* x, int64_t pixels, int32_t Cp, int32_t elem_bytes, const int32_t* idx, int32_t C,
                        void* out);

/* Largest absolute weight of every channel group (the criterion Sec. 4.1 describes next to the L2 one):
 * out_max[k] = max |w[k,:,:,:]|, in_max[c] = max |w[:,:,:,c]|. */
int oracle_group_maxabs(const double* w, int32_t K, int32_t RS, int32_t C, double* out_max, double* in_max);

/* Writes exact zeros into every weight of the flagged groups (Sec. 4.1: weights of a channel below the threshold
 * are zeroed out): w[k,:,:,c] = 0 where zero_out[k] or zero_in[c]; either mask may be NULL. */
int oracle_apply_zero(double* w, int32_t K, int32_t RS, int32_t C, const uint8_t* zero_out, const uint8_t* zero_in);

/* Optimizer step of Alg. 1 with the regulariser's gradient folded in, in place.  The paper names the step
 * (Optimizer(W, dW, LR)) and its ResNet baseline's hyper-parameters but not the rule; the reading used here
 * is stochastic gradient descent with momentum in its common form:
 *   g = dw + wd*w + lambda*w*(a/out_norm[k] + b/in_norm[c])   (a zero norm contributes 0)
 *   mom = mu*mom + g ;  w = w - lr*mom. */
int oracle_sgd_momentum_lasso(double* w, const double* dw, double* mom, const double* out_norm, const double* in_norm,
                              double lambda, double lr, double mu, double wd, uint32_t flags, int32_t K, int32_t RS,
                              int32_t C);

/* Feature (batch) normalisation over the N*H*W pixels of an NHWC tensor, training mode (Sec. 2.1: the
 * bandwidth-bound layers next to the convolutions; their cost scales with the compacted channel count):
 *   mean[c], var[c] = batch mean and biased variance of channel c;  invstd[c] = 1/sqrt(var[c] + eps);
 *   y[p,c] = (x[p,c] - mean[c]) * invstd[c] * gamma[c] + beta[c]. */
int oracle_bn_fwd(const double* x, int64_t pixels, int32_t C, const double* gamma, const double* beta, double eps,
                  double* y, double* mean, double* invstd);

/* Its gradients for an upstream gradient dy (the statistics depend on x):  xh = (x - mean)*invstd,
 *   dgamma[c] = sum_p dy*xh,  dbeta[c] = sum_p dy,
 *   dx[p,c] = gamma[c]*invstd[c] * (dy[p,c] - dbeta[c]/M - xh[p,c]*dgamma[c]/M),  M = pixels. */
int oracle_bn_bwd(const double* x, const double* dy, int64_t pixels, int32_t C, const double* gamma, const double* mean,
                  const double* invstd, double* dx, double* dgamma, double* dbeta);

#ifdef __cplusplus
}
#endif
#endif
