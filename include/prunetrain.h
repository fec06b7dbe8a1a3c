/*
 * prunetrain.h - C ABI of the MI355X (gfx950) PruneTrain conv-layer hot path.
 *
 * One training step of a convolution layer (forward, input gradient, weight gradient), the
 * channel-granular group-lasso regulariser (group norms and its gradient), and the periodic
 * reconfiguration pieces (zero-group detection, channel-edge reconciliation, compaction plan and
 * the compaction gathers), as the paper states them: Sec. 2.1 and Alg. 1 (ForwardProp / BackProp),
 * Eq. 4 (weight gradient), Eq. 1-2 (group lasso), Sec. 4.1 (threshold zeroing), Sec. 4.2
 * (adjacent-layer intersection, channel union, state carry-over at reconfiguration).
 *
 * Conventions
 *  - Every pointer named in a call is DEVICE memory owned by the caller unless the comment says
 *    "host".  The library never allocates, frees or retains memory and never synchronises: all
 *    work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the null stream) and
 *    buffers must stay valid until the stream has executed the call.
 *  - Layouts: activations NHWC  x[N][H][W][x_cpitch], y[N][P][Q][y_cpitch];
 *             weights     KRSC  w[K][R][S][w_cpitch].
 *    A `*_cpitch` is the physical length, in elements, of the innermost (channel) axis; it is
 *    >= the logical channel count.  Elements between the logical count and the pitch are never
 *    read as data, and are not written except where a call says so (pt_compact_nhwc, pt_bn_fwd /
 *    pt_bn_bwd, and the convolutions under PT_CONV_PAD_ZERO write zeros from the channel count up to
 *    the next multiple of 8).  Pitches that are multiples of 8 elements (16 bytes of
 *    bf16) select the vectorised kernels; any other pitch takes a slower element-wise path with
 *    identical results.
 *  - bf16 tensors are passed as uint16_t bit patterns (IEEE bfloat16, round-to-nearest-even on
 *    conversion from fp32).  Convolutions multiply bf16 inputs and accumulate in fp32.
 *  - Outputs are fully overwritten (logical elements only) except where a call says it accumulates.
 *    Inputs and outputs must not alias.
 *  - Every call returns a pt_status.  Argument errors are detected on the host before anything is
 *    enqueued.  No exception crosses this boundary.
 *  - State: none besides the last HIP error code and a one-time, idempotent opt-in of some kernels to
 *    large LDS allocations, made at their first launch on each device and recorded per device with
 *    atomics.  Calls may come from any host thread.
 */
#ifndef PRUNETRAIN_H
#define PRUNETRAIN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pt_status {
    PT_OK = 0,
    PT_ERR_NULL = -1,        /* a required pointer is NULL */
    PT_ERR_SHAPE = -2,       /* inconsistent descriptor: zero/negative extent, P/Q mismatch, pitch < extent */
    PT_ERR_WORKSPACE = -3,   /* workspace smaller than the matching *_workspace_bytes() */
    PT_ERR_UNSUPPORTED = -4, /* valid but outside this build's limits (see each call) */
    PT_ERR_LAUNCH = -5,      /* a HIP call failed; pt_last_hip_error() holds its code */
    PT_ERR_EMPTY = -6        /* pt_plan_layer_removal: an edge that is read outside the listed layers has died */
} pt_status;

/* Convolution problem: cross-correlation with zero padding, dilation 1, one group, no bias.
 * P = (H + 2*pad_h - R)/stride_h + 1, Q likewise; the call checks them. */
typedef struct pt_conv_desc {
    uint32_t struct_size; /* sizeof(pt_conv_desc), checked */
    int32_t N, H, W, C;   /* input  x[N][H][W][C] */
    int32_t K, R, S;      /* filter w[K][R][S][C] */
    int32_t stride_h, stride_w, pad_h, pad_w;
    int32_t P, Q;         /* output y[N][P][Q][K] */
    int32_t x_cpitch;     /* channel pitch of x and dx (>= C) */
    int32_t y_cpitch;     /* channel pitch of y and dy (>= K) */
    int32_t w_cpitch;     /* channel pitch of w (bf16) and of dw (fp32) (>= C) */
    uint32_t flags;       /* PT_CONV_* bits, 0 = none; unknown bits give PT_ERR_UNSUPPORTED */
} pt_conv_desc;

/* The caller vouches that the padding channels of the call's bf16 INPUT tensors hold zeros: c in [C, x_cpitch) of x,
 * k in [K, y_cpitch) of dy, c in [C, w_cpitch) of w.  Without the flag padding may hold anything (NaN included) and
 * the kernels clear it on the fly, which costs time whenever C (forward) or K (input gradient) is not a multiple
 * of 8.  Buffers that start out zeroed and are only ever written by this library keep zero padding: without the
 * flag no call writes padding channels, and with it pt_conv_fwd / pt_conv_bwd_data[_crsk] write only zeros there
 * (the last 8-channel chunk of y / dx goes out as one 16-byte store).  With the flag set and non-zero input
 * padding the results are undefined (never out of bounds). */
#define PT_CONV_PAD_ZERO 1u

/* Library version (major*10000 + minor*100 + patch) and the last failing HIP error code (0 if none). */
int32_t pt_version(void);
int32_t pt_last_hip_error(void);

/* ---- convolution: Sec. 2.1, Alg. 1 ForwardProp / BackProp, Eq. 4 ---------------------------- */

/* Host-only: bytes of workspace each convolution call needs for this descriptor (may be 0). */
int32_t pt_conv_fwd_workspace_bytes(const pt_conv_desc* d, size_t* bytes);
int32_t pt_conv_bwd_data_workspace_bytes(const pt_conv_desc* d, size_t* bytes);
int32_t pt_conv_bwd_weight_workspace_bytes(const pt_conv_desc* d, size_t* bytes);

/* y[n,p,q,k] = sum_{r,s,c} x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + s, c] * w[k,r,s,c].
 * x, w bf16; y bf16 (fp32 accumulator rounded once). ws: device scratch of ws_bytes (256-byte aligned).
 * An image-like first layer under PT_CONV_PAD_ZERO (C <= 4 at x_cpitch = w_cpitch = 8, y_cpitch a multiple of 8,
 * filter <= 8 x 8, stride 1 or 2, 16-byte aligned tensors) takes a kernel of its own, and so does a 3 x 3 filter at
 * stride 1 and padding 1 with at most 64 channels on either side (pitches multiples of 8, channel counts multiples
 * of 8 or PT_CONV_PAD_ZERO); same results to the same tolerance. */
int32_t pt_conv_fwd(const pt_conv_desc* d, const uint16_t* x, const uint16_t* w, uint16_t* y, void* ws,
                    size_t ws_bytes, void* stream);

/* n independent forward convolutions in one call (Sec. 2.1: e.g. the first convolution of a residual block and the
 * block's shortcut convolution, which read the same input and meet only at the block's output).  Same results as n
 * calls of pt_conv_fwd; problems that the direct kernel takes with the same instantiation share a launch, so the
 * tail of one overlaps the head of the next.  descs: host array of n descriptors; x, w, y: host arrays of n device
 * pointers each.  n <= 0 is an error (PT_ERR_SHAPE); any invalid descriptor or NULL pointer fails the whole call
 * before anything is launched. */
int32_t pt_conv_fwd_batched(const pt_conv_desc* descs, const uint16_t* const* x, const uint16_t* const* w,
                            uint16_t* const* y, int32_t n, void* stream);

/* dx = adjoint of the forward map in x applied to dy:
 * dx[n,h,w,c] = sum over (p,q,k,r,s) with p*stride_h - pad_h + r == h, q*stride_w - pad_w + s == w
 *               of dy[n,p,q,k] * w[k,r,s,c].   dy, w bf16; dx bf16, every logical element written
 * (zeros where no output pixel reads the input pixel). */
int32_t pt_conv_bwd_data(const pt_conv_desc* d, const uint16_t* dy, const uint16_t* w, uint16_t* dx, void* ws,
                         size_t ws_bytes, void* stream);

/* The input-gradient GEMM reduces over k, so it reads the filter bank with k innermost:
 *   wt[c][r][s][k] = w[k][r][s][c], bf16, k pitch = K rounded up to a multiple of 8 (padding written as 0).
 * pt_conv_bwd_data builds this copy in its workspace on every call.  A training step can instead convert
 * all layers once per iteration (the weights change once per iteration) with pt_weights_to_crsk_batched -
 * `layers` is a HOST array whose pointers are device pointers, wt 16-byte aligned - and call
 * pt_conv_bwd_data_crsk, which has the semantics of pt_conv_bwd_data and needs no workspace. */
typedef struct pt_layer_crsk {
    const uint16_t* w; /* [K][RS][w_cpitch] bf16 */
    uint16_t* wt;      /* [C][RS][round_up(K,8)] bf16 */
    int32_t K, RS, C, w_cpitch;
} pt_layer_crsk;
int32_t pt_weights_to_crsk_batched(const pt_layer_crsk* layers, int32_t n, void* stream);
int32_t pt_conv_bwd_data_crsk(const pt_conv_desc* d, const uint16_t* dy, const uint16_t* wt, uint16_t* dx,
                              void* stream);

/* dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + s, c]  (Eq. 4;
 * plain sum over the mini-batch).  x, dy bf16; dw fp32 [K][R][S][w_cpitch].  The reduction is split
 * over workgroups into ws and combined in a fixed order: results are run-to-run identical.  An image-like first
 * layer (C <= 4 at x_cpitch 8, K <= 64, filter <= 8 x 8, stride 1 or 2, 16-byte aligned x and dy) takes a kernel of
 * its own, which always writes one slab of partial sums per workgroup: ws must not be NULL there (the workspace query
 * says how much). */
int32_t pt_conv_bwd_weight(const pt_conv_desc* d, const uint16_t* x, const uint16_t* dy, float* dw, void* ws,
                           size_t ws_bytes, void* stream);

/* Host-only: how pt_conv_bwd_weight[_lasso] would run this descriptor on 16-byte aligned tensors (aligned != 0) or
 * on unaligned ones: the number of workgroup slices of the pixel reduction (1 = the main kernel writes dw itself),
 * output tiles per slice, and which pass combines the slices (PT_WGRAD_REDUCE_*).  The first layer's own kernel
 * reports its workgroups as slices of one tile, always combined by the deep pass.  For tests and tuning: lets a
 * caller assert that a problem size reaches the code path it is meant to cover. */
#define PT_WGRAD_REDUCE_NONE 0 /* unsplit: no second pass (with the regulariser: added in the main kernel's epilogue, or
                                  by a pass over one slab when the main kernel cannot) */
#define PT_WGRAD_REDUCE_DEEP 1 /* many slices over few outputs: one output per lane, slices spread over wavefronts */
#define PT_WGRAD_REDUCE_WIDE 2 /* few slices over many outputs: four outputs per thread, slices in ascending order */
typedef struct pt_wgrad_plan_info {
    int32_t splits, tiles, reduce_kind, tile_m, tile_n;
} pt_wgrad_plan_info;
int32_t pt_conv_bwd_weight_plan(const pt_conv_desc* d, int32_t aligned, pt_wgrad_plan_info* info);

/* ---- group lasso: Eq. 1-2 ------------------------------------------------------------------- */

/* Channel-group L2 norms of one layer's fp32 master weights w[K][RS][w_cpitch], RS = R*S:
 *   out_norm[k] = ||w[k,:,:]||_2 (filter k), in_norm[c] = ||w[:,:,c]||_2 (input channel c).
 * If w_shadow is not NULL it receives the bf16 copy of w (same shape and pitch) that the
 * convolutions consume, produced from the same single read of w.
 * Limit: C <= 2048.  A 16-byte aligned w with w_cpitch % 4 == 0 takes the vectorised path.
 * Deterministic (fixed reduction order).  ws: device scratch, 16-byte aligned. */
int32_t pt_group_norms_workspace_bytes(int32_t K, int32_t RS, int32_t C, size_t* bytes);
int32_t pt_group_norms(const float* w, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch, float* out_norm,
                       float* in_norm, uint16_t* w_shadow, void* ws, size_t ws_bytes, void* stream);

/* pt_group_norms for callers that cannot allocate device memory or bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  Same arguments minus the workspace, same kernels and
 * results; the scratch (row sums and per-chunk column partials) is an array of 4 MiB that the library holds on every
 * device it runs on, for as long as the process lives.  A layer whose pt_group_norms_workspace_bytes exceeds 4 MiB
 * is rejected with PT_ERR_WORKSPACE before anything is enqueued.  The call allocates and frees nothing, on the
 * device or through any library.  Nothing in the scratch needs clearing: every element a call reads it has written
 * itself.  All calls on one device share the one array: calls that overlap on a device (different streams, or
 * different host threads' streams) race; order them on one stream or with events. */
int32_t pt_group_norms_static(const float* w, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch, float* out_norm,
                              float* in_norm, uint16_t* w_shadow, void* stream);

/* Adds the gradient of lambda * (sum_k out_norm[k] + sum_c in_norm[c]) onto dw (accumulates):
 *   dw[k,rs,c] += lambda * w[k,rs,c] * (a / out_norm[k] + b / in_norm[c]),
 * a = flags bit 0 (regularise output groups), b = flags bit 1 (regularise input groups; clear it for
 * the network's first convolution, whose input groups are exempt).  A group whose norm is exactly 0
 * contributes 0.  dw has the shape and pitch of w. */
#define PT_LASSO_OUT 1u
#define PT_LASSO_IN 2u
int32_t pt_group_lasso_grad(const float* w, const float* out_norm, const float* in_norm, float lambda,
                            uint32_t flags, float* dw, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch,
                            void* stream);

/* Weight gradient with the regulariser's gradient folded in (Eq. 4 followed by the dW update of Alg. 1's GroupLassoReg
 * step): dw = pt_conv_bwd_weight's result + what pt_group_lasso_grad would add, written once - the pass that combines
 * the split partial sums adds the term, so dw is not written, read and rewritten.  w: the layer's fp32 master weights
 * [K][RS][w_cpitch]; out_norm [K], in_norm [C] as written by pt_group_norms for the same w; flags as above.  The
 * workspace is that of pt_conv_bwd_weight or one dw-sized slab, whichever is larger. */
int32_t pt_conv_bwd_weight_lasso_workspace_bytes(const pt_conv_desc* d, size_t* bytes);
int32_t pt_conv_bwd_weight_lasso(const pt_conv_desc* d, const uint16_t* x, const uint16_t* dy, const float* w,
                                 const float* out_norm, const float* in_norm, float lambda, uint32_t flags, float* dw,
                                 void* ws, size_t ws_bytes, void* stream);

/* Multi-layer forms: the regulariser of Eq. 2 runs over every layer of the network each iteration and a
 * layer's weights are small, so all layers go into a few launches (64 layers per launch pair for the norms, 32 per launch for the
 * gradient and the optimizer step).  `layers`
 * is a HOST array of n descriptors whose pointers are device pointers; per layer the semantics,
 * limits and determinism are those of the single-layer calls above.  The workspace is split between
 * the layers in array order. */
typedef struct pt_layer_weights {
    const float* w;      /* [K][RS][w_cpitch] fp32 master weights */
    float* out_norm;     /* [K] */
    float* in_norm;      /* [C] */
    uint16_t* w_shadow;  /* NULL or bf16 [K][RS][w_cpitch] */
    int32_t K, RS, C, w_cpitch;
} pt_layer_weights;
typedef struct pt_layer_lasso {
    const float* w;         /* [K][RS][w_cpitch] */
    const float* out_norm;  /* [K] */
    const float* in_norm;   /* [C] */
    float* dw;              /* [K][RS][w_cpitch], accumulated into */
    int32_t K, RS, C, w_cpitch;
    uint32_t flags;         /* PT_LASSO_OUT | PT_LASSO_IN */
    uint32_t reserved;
} pt_layer_lasso;
int32_t pt_group_norms_batched_workspace_bytes(const pt_layer_weights* layers, int32_t n, size_t* bytes);
int32_t pt_group_norms_batched(const pt_layer_weights* layers, int32_t n, void* ws, size_t ws_bytes, void* stream);

/* Group norms and zero-group detection in the same two launches (Eq. 2 + threshold zeroing of Sec. 4.1): per
 * layer, out_norm / in_norm as pt_group_norms writes them and zero_out[k] = (out_norm[k] < thr),
 * zero_in[c] = (in_norm[c] < thr), the comparison of pt_zero_groups on the fp32 norms (strict; thr <= 0 marks
 * nothing).  `layers` is a HOST array; all five pointers of a layer are required.  Workspace as for
 * pt_group_norms_batched. */
typedef struct pt_layer_detect {
    const float* w;     /* [K][RS][w_cpitch] fp32 master weights */
    float* out_norm;    /* [K] */
    float* in_norm;     /* [C] */
    uint8_t* zero_out;  /* [K] */
    uint8_t* zero_in;   /* [C] */
    int32_t K, RS, C, w_cpitch;
} pt_layer_detect;
int32_t pt_group_norms_detect_batched_workspace_bytes(const pt_layer_detect* layers, int32_t n, size_t* bytes);
int32_t pt_group_norms_detect_batched(const pt_layer_detect* layers, int32_t n, float thr, void* ws, size_t ws_bytes,
                                      void* stream);
int32_t pt_group_lasso_grad_batched(const pt_layer_lasso* layers, int32_t n, float lambda, void* stream);

/* Optimizer step of Alg. 1 with the regulariser's gradient folded in (one pass over w, dw, mom instead of a
 * gradient pass plus an update pass).  The paper names the step but not the rule; this is stochastic gradient
 * descent with momentum in its common form, per layer and in place:
 *   g = dw + weight_decay*w + lambda*w*(a/out_norm[k] + b/in_norm[c])     (a zero norm contributes 0)
 *   mom = momentum*mom + g ;   w = w - lr*mom.
 * dw is the loss gradient WITHOUT the regulariser (what pt_conv_bwd_weight wrote) and is not modified; the norms
 * are those of the weights before the step.  `layers`: HOST array, device pointers inside; any n (32 layers per launch). */
typedef struct pt_layer_update {
    float* w;              /* [K][RS][w_cpitch] */
    const float* dw;       /* same shape */
    float* mom;            /* same shape */
    const float* out_norm; /* [K] */
    const float* in_norm;  /* [C] */
    int32_t K, RS, C, w_cpitch;
    uint32_t flags;        /* PT_LASSO_OUT | PT_LASSO_IN */
    uint32_t reserved;
} pt_layer_update;
int32_t pt_sgd_momentum_lasso_batched(const pt_layer_update* layers, int32_t n, float lambda, float lr, float momentum,
                                      float weight_decay, void* stream);

/* Value of the regulariser over a whole network (GroupLassoReg of Alg. 1, Eq. 1-2):
 *   *penalty_dev = sum over layers of ( a * sum_k out_norm[k] + b * sum_c in_norm[c] ),  a, b = flags bits.
 * No weighting by group size (one global coefficient, Sec. 4.1).  The norms are those pt_group_norms wrote;
 * `layers` is a HOST array whose pointers are device pointers; penalty_dev is a device double, overwritten
 * (0 for n == 0).  fp64 accumulation in a fixed order: run-to-run identical.  One small launch per 96 layers. */
typedef struct pt_layer_penalty {
    const float* out_norm; /* [K] */
    const float* in_norm;  /* [C] */
    int32_t K, C;
    uint32_t flags;        /* PT_LASSO_OUT | PT_LASSO_IN */
    uint32_t reserved;
} pt_layer_penalty;
int32_t pt_group_lasso_penalty_batched(const pt_layer_penalty* layers, int32_t n, double* penalty_dev, void* stream);

/* Host-only: SetCoeff of Alg. 1.  The coefficient for which the regulariser makes up `ratio` of the total loss at
 * the first iteration (penalty-ratio equation of Sec. 4.1; the paper uses 0.20-0.25):
 *   ratio = lambda*loss2 / (loss1 + lambda*loss2)   =>   lambda = ratio*loss1 / ((1 - ratio)*loss2),
 * loss1 = classification loss, loss2 = the value above.  PT_ERR_SHAPE unless 0 < ratio < 1, loss2 > 0, loss1 >= 0. */
int32_t pt_lasso_set_coeff(double loss1, double loss2, double ratio, double* lambda);

/* ---- reconfiguration: Sec. 4.1-4.2 ---------------------------------------------------------- */

/* zero[g] = (norms[g] < thr) ? 1 : 0, compared in fp32; thr <= 0 marks nothing. n may be 0. */
int32_t pt_zero_groups(const float* norms, int32_t n, float thr, uint8_t* zero, void* stream);

/* One channel edge: the output dimension of n_prod producer convolutions and the input dimension of
 * n_cons consumer convolutions must stay equal.  keep[j] = 0 only when channel j is zero in EVERY
 * producer's output mask and EVERY consumer's input mask (adjacent-layer intersection for 1+1,
 * channel union for a residual stage).  producer_zero / consumer_zero are HOST arrays of device
 * pointers to n-element masks; n_prod + n_cons must be in [1, 64]. */
int32_t pt_reconcile_edge(const uint8_t* const* producer_zero, int32_t n_prod, const uint8_t* const* consumer_zero,
                          int32_t n_cons, int32_t n, uint8_t* keep, void* stream);

/* idx[0 .. *n_keep) = ascending positions j with keep[j] != 0 (exclusive prefix sum of the mask);
 * idx must hold n entries; *n_keep_dev is written on the device (read it after synchronising). */
int32_t pt_compact_plan(const uint8_t* keep, int32_t n, int32_t* idx, int32_t* n_keep_dev, void* stream);

/* w_out[k'][rs][c'] = w[idxK[k']][rs][idxC[c']] for fp32 tensors (weights, their momentum).  A NULL index
 * list is the identity on that axis (then Kp == K / Cp == C).  Index values must lie inside the source. */
int32_t pt_compact_weights(const float* w, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch, const int32_t* idxK,
                           int32_t Kp, const int32_t* idxC, int32_t Cp, float* w_out, int32_t out_cpitch,
                           void* stream);

/* out[j'] = v[idx[j']] for per-channel vectors (bias, normalisation scale/shift/statistics, momentum);
 * elem_bytes in {1, 2, 4, 8}. n_keep may be 0. */
int32_t pt_compact_vector(const void* v, int32_t elem_bytes, const int32_t* idx, int32_t n_keep, void* out,
                          void* stream);

/* Multi-job forms of the four small reconfiguration steps.  A network has dozens of layers and channel
 * edges and each step on one of them is far below a launch's fixed cost, so whole-network tables go into
 * a handful of launches.  Every `jobs` / `edges` array is a HOST array whose pointers are device
 * pointers (except the member lists, which are host arrays of device pointers as in pt_reconcile_edge);
 * per job the semantics, limits and error rules are those of the single calls above.  Jobs of one call
 * must not write overlapping memory. */
typedef struct pt_norm_mask {
    const float* norms; /* [n] */
    uint8_t* zero;      /* [n] */
    int32_t n;
    int32_t reserved;
} pt_norm_mask;
int32_t pt_zero_groups_batched(const pt_norm_mask* jobs, int32_t n_jobs, float thr, void* stream);

/* pt_reconcile_edge followed by pt_compact_plan on the same edge, one workgroup per edge. */
typedef struct pt_edge_plan {
    const uint8_t* const* producer_zero; /* host array of n_prod device pointers */
    const uint8_t* const* consumer_zero; /* host array of n_cons device pointers */
    int32_t n_prod, n_cons;              /* n_prod + n_cons in [1, 64] */
    int32_t n;                           /* channels on this edge */
    int32_t reserved;
    uint8_t* keep;                       /* [n] */
    int32_t* idx;                        /* [n] */
    int32_t* n_keep_dev;                 /* device scalar */
} pt_edge_plan;
int32_t pt_reconcile_plan_batched(const pt_edge_plan* edges, int32_t n_edges, void* stream);

typedef struct pt_gather_vector {
    const void* v;
    const int32_t* idx;
    void* out;
    int32_t n_keep;
    int32_t elem_bytes; /* 1, 2, 4 or 8 */
} pt_gather_vector;
int32_t pt_compact_vector_batched(const pt_gather_vector* jobs, int32_t n_jobs, void* stream);

typedef struct pt_gather_weights {
    const float* w;      /* [K][RS][w_cpitch] */
    const int32_t* idxK; /* NULL = identity */
    const int32_t* idxC; /* NULL = identity */
    float* w_out;        /* [Kp][RS][out_cpitch] */
    int32_t K, RS, C, w_cpitch, Kp, Cp, out_cpitch;
    int32_t reserved;
} pt_gather_weights;
int32_t pt_compact_weights_batched(const pt_gather_weights* jobs, int32_t n_jobs, void* stream);

/* out[pix][c'] = x[pix][idx[c']] for bf16 NHWC activations with `pixels` = N*H*W rows.  Padding channels of out:
 * those from Cp up to the next multiple of 8 (as far as they lie inside out_cpitch) are written as zero, so that
 * rows are written whole and a convolution reading the result may be given PT_CONV_PAD_ZERO when out_cpitch is Cp
 * rounded up to 8; channels beyond that multiple of 8 are left untouched. */
int32_t pt_compact_nhwc(const uint16_t* x, int64_t pixels, int32_t C, int32_t x_cpitch, const int32_t* idx,
                        int32_t Cp, uint16_t* out, int32_t out_cpitch, void* stream);

/* Several activation tensors in one call (jobs: HOST array, device pointers inside; per job the semantics of
 * pt_compact_nhwc).  Tensors with 16-byte aligned rows share launches of the streaming kernel. */
typedef struct pt_gather_nhwc {
    const uint16_t* x;
    const int32_t* idx;
    uint16_t* out;
    int64_t pixels;
    int32_t C, x_cpitch, Cp, out_cpitch;
} pt_gather_nhwc;
int32_t pt_compact_nhwc_batched(const pt_gather_nhwc* jobs, int32_t n_jobs, void* stream);

/* ---- channel gating pieces and the paper's other zeroing rule: Sec. 4.1, 4.2 ----------------------------- */

/* Channel scatter, the inverse of pt_compact_nhwc (the scatter layer of channel gating, Sec. 4.2):
 *   out[pix][idx[c']] = x[pix][c'] for c' < Cp; every other logical channel of out is written as zero.
 * x has Cp channels at pitch x_cpitch, out has C channels at pitch out_cpitch; idx as written by pt_compact_plan
 * (strictly ascending, values < C).  Limit: C <= 8192. */
int32_t pt_scatter_nhwc(const uint16_t* x, int64_t pixels, int32_t Cp, int32_t x_cpitch, const int32_t* idx, int32_t C,
                        uint16_t* out, int32_t out_cpitch, void* stream);

/* Largest absolute weight per channel group (Sec. 4.2 states the zeroing rule this way):
 *   out_max[k] = max |w[k,:,:]|,  in_max[c] = max |w[:,:,c]|.   Exact (a maximum has no rounding); feed the
 * results to pt_zero_groups like norms.  Limit: C <= 2048.  Three small launches. */
int32_t pt_group_maxabs(const float* w, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch, float* out_max,
                        float* in_max, void* stream);

/* Writes exact zeros into the flagged groups of an fp32 [K][RS][w_cpitch] tensor (weights, momentum):
 *   w[k][rs][c] = 0 where zero_out[k] != 0 or zero_in[c] != 0.   Either mask may be NULL (none of that kind). */
int32_t pt_apply_zero(float* w, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch, const uint8_t* zero_out,
                      const uint8_t* zero_in, void* stream);

/* ---- feature normalisation next to the convolutions: Sec. 2.1 (the bandwidth-bound layers) ------------------ */

/* Training-mode normalisation of a bf16 NHWC tensor over its `pixels` = N*H*W rows, per channel:
 *   mean[c] = sum_p x[p][c] / pixels,  var[c] = sum_p (x[p][c] - mean[c])^2 / pixels  (biased),
 *   invstd[c] = 1 / sqrt(var[c] + eps),  y[p][c] = bf16((x[p][c] - mean[c]) * invstd[c] * gamma[c] + beta[c]).
 * x, y: device, rows of x_cpitch / y_cpitch elements, both multiples of 8 and >= C, 16-byte aligned bases; channels
 * >= C of a row are never read into a result.  Of y's padding, the channels from C up to the next multiple of 8 are
 * written as zero (rows go out as whole 16-byte vectors, and a convolution reading y may be given
 * PT_CONV_PAD_ZERO when y_cpitch is C rounded up to 8); channels beyond are left untouched.  gamma, beta: device fp32 [C] (inputs); mean, invstd:
 * device fp32 [C] (outputs, kept by the caller for pt_bn_bwd).  ws: device scratch of pt_bn_workspace_bytes().
 * Statistics are combined in fp64 in a fixed order: run-to-run identical.  Three launches on `stream`.
 * Limits: C <= 2048, pixels < 2^31 (else PT_ERR_UNSUPPORTED; so are pitches that are not multiples of 8). */
int32_t pt_bn_workspace_bytes(int64_t pixels, int32_t C, size_t* bytes);
int32_t pt_bn_fwd(const uint16_t* x, int64_t pixels, int32_t C, int32_t x_cpitch, const float* gamma,
                  const float* beta, float eps, uint16_t* y, int32_t y_cpitch, float* mean, float* invstd, void* ws,
                  size_t ws_bytes, void* stream);

/* Backward of pt_bn_fwd given dy (bf16, same shape, pitch dy_cpitch) and the forward's mean / invstd:
 *   xhat = (x - mean) * invstd,  dbeta[c] = sum_p dy[p][c],  dgamma[c] = sum_p dy[p][c] * xhat[p][c],
 *   dx[p][c] = bf16(gamma[c] * invstd[c] * (dy[p][c] - dbeta[c]/pixels - xhat[p][c] * dgamma[c]/pixels)).
 * dgamma, dbeta: device fp32 [C] outputs.  Same layout rules (dx's padding like y's), limits and workspace as
 * pt_bn_fwd. */
int32_t pt_bn_bwd(const uint16_t* x, const uint16_t* dy, int64_t pixels, int32_t C, int32_t x_cpitch,
                  int32_t dy_cpitch, const float* gamma, const float* mean, const float* invstd, uint16_t* dx,
                  int32_t dx_cpitch, float* dgamma, float* dbeta, void* ws, size_t ws_bytes, void* stream);

/* Forward convolution that also reduces its output for the normalisation layer behind it (Sec. 2.1 notes that these
 * layers read their input several times; this removes one of the reads).  Same y as pt_conv_fwd; in addition
 * `sums` (device, fp32) receives, per tile of 128 output pixels, the per-channel sums of the STORED outputs (the
 * bf16-rounded values) and of their squares: sums[(q * n_partial + t) * K + k], q = 0 / 1.  The workspace query
 * returns the size of `sums` and n_partial.  pt_bn_fwd_from_sums then finishes the statistics (fp64, fixed order)
 * and normalises: the results of pt_bn_fwd up to the summation order (the sums are taken about 0, not about a
 * pivot, so a channel whose mean is large against its spread loses the digits it would lose in any one-pass
 * variance).  PT_ERR_UNSUPPORTED when the layer does not take the direct kernel: pitches not multiples of 8 or bases
 * not 16-byte aligned, more than 64 filter taps, or C not a multiple of 8 without PT_CONV_PAD_ZERO. */
int32_t pt_conv_fwd_stats_workspace_bytes(const pt_conv_desc* d, size_t* bytes, int32_t* n_partial);
int32_t pt_conv_fwd_stats(const pt_conv_desc* d, const uint16_t* x, const uint16_t* w, uint16_t* y, float* sums,
                          size_t sums_bytes, void* stream);
int32_t pt_bn_fwd_from_sums(const uint16_t* x, int64_t pixels, int32_t C, int32_t x_cpitch, const float* sums,
                            int32_t n_partial, const float* gamma, const float* beta, float eps, uint16_t* y,
                            int32_t y_cpitch, float* mean, float* invstd, void* stream);

/* ---- layer removal: Sec. 4.1 ("Layer Removal by Overlapping Regularization Groups") --------------------------- */

/* HOST-only graph logic, no device work.  After a plan, an edge with no survivors (n_keep == 0) carries nothing: the
 * layers writing it and the layers reading it are removed.  Removal propagates: an edge all of whose producers are
 * removed carries nothing, an edge all of whose consumers are removed is read by nobody - unless it is also fed
 * (PT_EDGE_FED_OUTSIDE: the network input, an identity shortcut from elsewhere) or read (PT_EDGE_READ_OUTSIDE: the
 * classifier behind the last stage) outside the listed layers.  An edge with no listed producers counts as fed, one
 * with no listed consumers as read.  removed_layers[n_layers] and dead_edges[n_edges] (host, 0/1) receive the fixed
 * point.  Returns PT_ERR_EMPTY (outputs still filled) if an edge that is read outside has died: the network is cut.
 * In a residual network the result is whole branches taken out with the shortcut left in place. */
#define PT_EDGE_FED_OUTSIDE 1
#define PT_EDGE_READ_OUTSIDE 2
typedef struct pt_removal_edge {
    const int32_t* producers; /* host: ids of the layers whose output channels are this edge */
    const int32_t* consumers; /* host: ids of the layers whose input channels are this edge */
    int32_t n_prod, n_cons;
    int32_t n_keep;           /* survivors in the latest plan (host copy of the plan's device count) */
    int32_t external;         /* PT_EDGE_* bits */
} pt_removal_edge;
int32_t pt_plan_layer_removal(const pt_removal_edge* edges, int32_t n_edges, int32_t n_layers, uint8_t* removed_layers,
                              uint8_t* dead_edges);

#ifdef __cplusplus
}
#endif
#endif
