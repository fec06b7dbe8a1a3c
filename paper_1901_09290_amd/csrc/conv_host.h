// Host-side planning of the convolution launches: descriptor checks, kernel argument construction,
// tile-configuration choice and the split plan of the weight gradient.
#pragma once

#include "conv_kernels.h"

namespace pt {

inline int32_t check_desc(const pt_conv_desc* d) {
    if (!d) return PT_ERR_NULL;
    if (d->struct_size != sizeof(pt_conv_desc)) return PT_ERR_SHAPE;
    if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0) return PT_ERR_SHAPE;
    if (d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0) return PT_ERR_SHAPE;
    if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S) return PT_ERR_SHAPE;
    if (d->P != (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1) return PT_ERR_SHAPE;
    if (d->Q != (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1) return PT_ERR_SHAPE;
    if (d->x_cpitch < d->C || d->y_cpitch < d->K || d->w_cpitch < d->C) return PT_ERR_SHAPE;
    if (d->flags & ~PT_CONV_PAD_ZERO) return PT_ERR_UNSUPPORTED;
    // limits of the 16/32-bit pixel arithmetic inside the kernels
    if (d->H > 16384 || d->W > 16384 || d->R > 255 || d->S > 255 || d->pad_h > 255 || d->pad_w > 255 ||
        d->stride_h > 255 || d->stride_w > 255)
        return PT_ERR_UNSUPPORTED;
    const int64_t in_pix = (int64_t)d->N * d->H * d->W, out_pix = (int64_t)d->N * d->P * d->Q;
    if (in_pix >= (1ll << 30) || out_pix >= (1ll << 30)) return PT_ERR_UNSUPPORTED;
    const int64_t big = d->H > d->W ? d->H : d->W;  // divisors of the in-kernel pixel decompositions
    if (in_pix * big >= (1ll << 32) || out_pix * big >= (1ll << 32)) return PT_ERR_UNSUPPORTED;
    // 32-bit element offsets into every tensor
    // (a margin below 2^31 elements: the buffer addressing of the direct kernels shifts offsets by up to a padded border)
    if (in_pix * d->x_cpitch >= (1ll << 31) - (1ll << 27) || out_pix * d->y_cpitch >= (1ll << 31) - (1ll << 27)) return PT_ERR_UNSUPPORTED;
    if ((int64_t)d->K * d->R * d->S * d->w_cpitch >= (1ll << 31)) return PT_ERR_UNSUPPORTED;
    if ((int64_t)d->C * d->R * d->S * round_up(d->K, 8) >= (1ll << 31)) return PT_ERR_UNSUPPORTED;
    if ((int64_t)d->R * d->S * round_up(d->C, 8) >= (1ll << 30)) return PT_ERR_UNSUPPORTED;
    if ((int64_t)d->R * d->S * round_up(d->K, 8) >= (1ll << 30)) return PT_ERR_UNSUPPORTED;
    return PT_OK;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

inline IgemmArgs make_fwd_args(const pt_conv_desc* d, const uint16_t* x, const uint16_t* w, uint16_t* y) {
    IgemmArgs a{};
    a.A = x; a.B = w; a.D = y;
    a.pad_zero = (d->flags & PT_CONV_PAD_ZERO) != 0;
    a.zf_h = a.zf_w = 1;
    a.M = d->N * d->P * d->Q;
    a.gW = make_fastdiv((uint32_t)d->Q); a.gH = make_fastdiv((uint32_t)d->P);
    a.srcH = d->H; a.srcW = d->W; a.apitch = d->x_cpitch;
    a.h_mul = d->stride_h; a.h_add = -d->pad_h; a.w_mul = d->stride_w; a.w_add = -d->pad_w;
    a.tr_step = 1; a.ts_step = 1; a.TR = d->R; a.TS = d->S;
    a.Cred = d->C; a.CredP = (int)round_up(d->C, 8);
    a.b_tap0 = 0; a.b_tr_stride = d->S; a.b_ts_stride = 1; a.b_taps = d->R * d->S;
    a.bpitch = d->w_cpitch; a.Nout = d->K;
    a.DH = d->P; a.DW = d->Q; a.d_hmul = 1; a.d_hadd = 0; a.d_wmul = 1; a.d_wadd = 0; a.dpitch = d->y_cpitch;
    a.d_linear = 1;
    a.fold = 0; a.TSm = d->S; a.Creal = d->C; a.Cfold = make_fastdiv((uint32_t)a.CredP);
    a.d_vec = (d->y_cpitch % 4 == 0) && (((uintptr_t)y & 7) == 0);
    a.d_vec16 = (d->y_cpitch % 8 == 0) && aligned16(y);
    return a;
}

// One stride-parity class (ca, cb) of input pixels of the input-gradient problem: the pixels
// h = ca + stride_h*i, w = cb + stride_w*j, reached only by taps r = r0 + stride_h*jr, s = s0 + stride_w*js.
struct BwdClass {
    int gH, gW, r0, s0, TR, TS;
};

inline BwdClass bwd_data_class(const pt_conv_desc* d, int ca, int cb) {
    BwdClass c;
    c.gH = ca < d->H ? (d->H - ca + d->stride_h - 1) / d->stride_h : 0;
    c.gW = cb < d->W ? (d->W - cb + d->stride_w - 1) / d->stride_w : 0;
    c.r0 = (ca + d->pad_h) % d->stride_h;
    c.s0 = (cb + d->pad_w) % d->stride_w;
    c.TR = c.r0 < d->R ? (d->R - c.r0 + d->stride_h - 1) / d->stride_h : 0;
    c.TS = c.s0 < d->S ? (d->S - c.s0 + d->stride_w - 1) / d->stride_w : 0;
    return c;
}

inline IgemmArgs make_bwd_data_args(const pt_conv_desc* d, const BwdClass& c, int ca, int cb, const uint16_t* dy,
                                    const uint16_t* wt, uint16_t* dx) {
    const int kpitch = (int)round_up(d->K, 8);
    IgemmArgs a{};
    a.A = dy; a.B = wt; a.D = dx;
    a.pad_zero = (d->flags & PT_CONV_PAD_ZERO) != 0;  // the k-innermost weight copy always has zero padding
    a.zf_h = a.zf_w = 1;
    a.M = d->N * c.gH * c.gW;
    a.gW = make_fastdiv((uint32_t)c.gW); a.gH = make_fastdiv((uint32_t)c.gH);
    a.srcH = d->P; a.srcW = d->Q; a.apitch = d->y_cpitch;
    a.h_mul = 1; a.h_add = (ca + d->pad_h - c.r0) / d->stride_h;
    a.w_mul = 1; a.w_add = (cb + d->pad_w - c.s0) / d->stride_w;
    a.tr_step = -1; a.ts_step = -1; a.TR = c.TR; a.TS = c.TS;
    a.Cred = d->K; a.CredP = kpitch;
    a.b_tap0 = c.r0 * d->S + c.s0; a.b_tr_stride = d->stride_h * d->S; a.b_ts_stride = d->stride_w;
    a.b_taps = d->R * d->S; a.bpitch = kpitch; a.Nout = d->C;
    a.DH = d->H; a.DW = d->W; a.d_hmul = d->stride_h; a.d_hadd = ca; a.d_wmul = d->stride_w; a.d_wadd = cb;
    a.dpitch = d->x_cpitch;
    a.d_linear = (d->stride_h == 1 && d->stride_w == 1);
    a.fold = 0; a.TSm = c.TS; a.Creal = d->K; a.Cfold = make_fastdiv((uint32_t)kpitch);
    a.d_vec = (d->x_cpitch % 4 == 0) && (((uintptr_t)dx & 7) == 0);
    a.d_vec16 = (d->x_cpitch % 8 == 0) && aligned16(dx);
#ifndef PT_BWD_EDGE_PRIO
#define PT_BWD_EDGE_PRIO 2
#endif
    a.edge_prio = PT_BWD_EDGE_PRIO;
    return a;
}

// Kernel and tile configuration.  `vec`: all operand rows are 16-byte aligned (pitches are multiples of 8
// elements) - then the direct global->LDS kernel is used, with a tall pixel tile for narrow outputs.
// Unaligned pitches, and filters with more than 64 taps per launch (the direct kernel keeps one validity
// bit per tap in a 64-bit mask), take the register-staged kernel.
// `plan` == nullptr: the problem is launched.  Otherwise, when the direct kernel takes it, nothing is launched yet: the
// plan is filled in and *planned set, for launch_igemm_dl_planned to send it out together with other problems (the
// register-staged kernel is launched at once either way, *planned cleared).
inline hipError_t launch_igemm(IgemmArgs& a, bool vec, hipStream_t st, IgemmDlPlan* plan = nullptr, bool* planned = nullptr) {
    if (planned) *planned = false;
    if (!vec) return launch_igemm_cfg<128, 128, 32, 2, 2, 2, 2, false>(a, st);
    // Small dense channel counts (an image-like input): fold the S taps of a filter row into one run
    if (a.CredP < 64 && a.TS > 1 && a.ts_step == 1 && a.apitch == a.CredP && a.bpitch == a.CredP && a.b_ts_stride == 1 &&
        a.TR * a.TS <= 64) {
        a.fold = 1;
        a.TSm = a.TS;
        a.Creal = a.Cred;
        a.Cfold = make_fastdiv((uint32_t)a.CredP);
        a.Cred = a.CredP = a.TS * a.CredP;
        a.TS = 1;
    }
    if (a.TR * a.TSm > 64) return launch_igemm_cfg<128, 128, 32, 2, 2, 2, 2, true>(a, st);
    // 128x128 tiles when they still fill the chip, else 128x64 tiles (more workgroups, deeper pipeline)
    const int64_t tiles128 = ceil_div(a.M, 128) * ceil_div(a.Nout, 128);
    // very many pixel tiles and a narrow output (the stem): tall tiles, so half as many workgroups pay set-up and fill
    IgemmDlPlan own;
    IgemmDlPlan& p = plan ? *plan : own;
    hipError_t e;
    if (a.Nout <= 64 && tiles128 >= 4096 && !a.stats) e = plan_igemm_dl_cfg<256, 64, 4, 2, 2>(a, p);
    else if (a.Nout <= 64 || tiles128 < 256) e = plan_igemm_dl_cfg<128, 64, 4, 2, 3>(a, p);
    else e = plan_igemm_dl_cfg<128, 128, 2, 4, 2>(a, p);
    if (e != hipSuccess) return e;
    if (plan) {
        *planned = true;
        return hipSuccess;
    }
    return launch_igemm_dl_planned(&a, &p, 1, st);
}

inline size_t bwd_data_ws(const pt_conv_desc* d) {
    return (size_t)round_up((int64_t)d->C * d->R * d->S * round_up(d->K, 8) * 2, 256);
}

// Split plan of the weight gradient.  `dl`: the direct global->LDS kernel (one filter tap per tile row
// block, tiles of 64 or 128 channels) is used; otherwise the register-staged kernel (flattened
// (tap, channel) axis, fixed 128x128 tiles).
struct WgradPlan {
    int dl, fold, BM, BN;
    int bkp;  // direct kernel: output pixels per reduction step
    int splits, iters_total, iters_per_split, tiles_m, tiles_n, tiles_per_tap, CP, KP, Mtot;
    size_t ws_bytes;
};
constexpr int kWgBM = 128, kWgBN = 128, kWgBK = 32;  // register-staged kernel
constexpr int kWgDlBKP = 64;                          // direct kernel: pixels per reduction step
// The same for 128 x 128 tiles: 32 pixels, five stages deep = 80 KB of LDS.  A step of 64 pixels at three stages
// (96 KB) is 4 % faster when the kernel runs alone, but a workgroup of that size shares a CU's 160 KB with no
// workgroup of the input-gradient kernel's three-stage form (72 KB) and only just with its two-stage form (64 KB);
// weight gradients are meant to run beside the input-gradient chain, and there the smaller footprint wins: full-width
// train step -2.2 %, pruned +0.6 % (A/B on one box, three runs each; 64 KB in four stages: -1.9 % / +0.9 %).
constexpr int kWgDlBKPBig = 32;
// Workgroups per launch the split count aims at (128x128 tiles: kWgTargetBlocksBig).  Well below the 512 resident
// slots on purpose: weight gradients of different layers are independent and are meant to run side by side on
// several streams, so one launch need not fill the chip, and every split costs a tile of fp32 partial sums written
// and read again.  Measured on the ResNet-50 step with four side streams: 512/256 -> 245, 256/96 -> 264 TFLOP/s
// (run one after the other on a single stream the same launches are ~25 % slower than with 512/256).  Later, with
// the first layer on a kernel of its own, A/B in one process (train step at full + pruned width, two runs each):
// 256/96 6.29 ms, 192/96 6.24, 160/96 6.23, 128/96 6.26, 192/112 6.29, 160/112 6.28, 320/96 6.37, 256/80 6.40,
// 256/128 6.39 - although the weight-gradient family called one after the other is fastest at 256/128 (1.79 vs
// 2.09 ms at full width): fewer, longer workgroups leave the input-gradient chain more of the chip.
#ifndef PT_WG_TARGET_SMALL
#define PT_WG_TARGET_SMALL 160
#endif
#ifndef PT_WG_TARGET_BIG
#define PT_WG_TARGET_BIG 96
#endif
constexpr int kWgTargetBlocks = PT_WG_TARGET_SMALL, kWgTargetBlocksBig = PT_WG_TARGET_BIG;
constexpr int kWgTargetAlone = 512;  // a launch known to run by itself: one resident round of the small tiles

// 64-wide tiles when 128-wide ones would waste more than ~20 % of their rows
inline int pick_tile(int n) {
    const int64_t r128 = round_up(n, 128), r64 = round_up(n, 64);
    return (r64 < r128 && r128 * 5 > (int64_t)n * 6) ? 64 : 128;
}

inline WgradPlan plan_wgrad(const pt_conv_desc* d, bool dl) {
    WgradPlan p;
    p.dl = dl;
    p.CP = (int)round_up(d->C, 8);
    p.KP = (int)round_up(d->K, 8);
    p.Mtot = d->R * d->S * p.CP;
    const int64_t pixels = (int64_t)d->N * d->P * d->Q;
    p.fold = dl && p.CP < 64 && d->S > 1 && d->x_cpitch == p.CP && d->w_cpitch == p.CP;
    if (dl) {
        const int run = p.fold ? d->S * p.CP : p.CP;  // contiguous elements of one tile row block
        p.BM = pick_tile(run);
        p.BN = pick_tile(p.KP);
        p.tiles_per_tap = (int)ceil_div(run, p.BM);
        p.tiles_m = (p.fold ? d->R : d->R * d->S) * p.tiles_per_tap;
        p.tiles_n = (int)ceil_div(d->K, p.BN);
        p.bkp = (p.BM == 128 && p.BN == 128) ? kWgDlBKPBig : kWgDlBKP;
        p.iters_total = (int)ceil_div(pixels, p.bkp);
    } else {
        p.bkp = kWgBK;
        p.BM = kWgBM;
        p.BN = kWgBN;
        p.tiles_per_tap = 0;
        p.tiles_m = (int)ceil_div(p.Mtot, kWgBM);
        p.tiles_n = (int)ceil_div(d->K, kWgBN);
        p.iters_total = (int)ceil_div(pixels, kWgBK);
    }
    // At least 4 reduction steps per workgroup.
    const int tiles = p.tiles_m * p.tiles_n;
    // Folded (image-like) inputs belong to a network's first layer, whose weight gradient is the last kernel of a
    // backward pass and runs when nothing is left to run beside it: that one fills the chip (train step -0.7 %).
    const int target = p.fold ? kWgTargetAlone : (dl && p.BM == 128 && p.BN == 128) ? kWgTargetBlocksBig : kWgTargetBlocks;
    int64_t splits = target / tiles;
    const int64_t max_splits = p.iters_total / 4 > 0 ? p.iters_total / 4 : 1;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    p.iters_per_split = (int)ceil_div(p.iters_total, splits);
    p.splits = (int)ceil_div(p.iters_total, p.iters_per_split);
    p.ws_bytes = p.splits > 1 ? (size_t)round_up((int64_t)p.splits * d->K * p.Mtot * 4, 256) : 0;
    return p;
}

// The resident-weights kernel takes 3 x 3 filters at stride 1 and padding 1 with at most 64 channels on either side,
// 16-byte aligned rows, and channel counts that are multiples of 8 or the caller's PT_CONV_PAD_ZERO (the padding of the
// operand it reduces over must be zero, and it writes the output's last chunk whole, zeros in its padding).
// PT_RES3: bit 0 = forward calls, bit 1 = input-gradient calls, bit 2 = those of any filter bank size.
#ifndef PT_RES3
#define PT_RES3 3
#endif
constexpr int kRes3BwdMaxBank = 3072;  // K * C up to which an input-gradient call takes the kernel
inline bool res3_shape_ok(const pt_conv_desc* d) {
    return d->R == 3 && d->S == 3 && d->stride_h == 1 && d->stride_w == 1 && d->pad_h == 1 && d->pad_w == 1 && d->C <= 64 &&
           d->K <= 64 && d->x_cpitch % 8 == 0 && d->y_cpitch % 8 == 0 &&
           (int64_t)d->H * d->W * (d->x_cpitch > d->y_cpitch ? d->x_cpitch : d->y_cpitch) * 2 <= 0x7fffffff;
}
inline bool res3_fwd_ok(const pt_conv_desc* d, const uint16_t* x, const uint16_t* w, const uint16_t* y) {
    return (PT_RES3 & 1) && res3_shape_ok(d) && d->w_cpitch % 8 == 0 && aligned16(x) && aligned16(w) && aligned16(y) &&
           ((d->C % 8 == 0 && d->K % 8 == 0) || (d->flags & PT_CONV_PAD_ZERO));
}
inline bool res3_bwd_ok(const pt_conv_desc* d, const uint16_t* dy, const uint16_t* wt, const uint16_t* dx) {
    // (input-gradient launches share the chip with weight gradients on other streams, and a workgroup that holds a CU's
    // whole LDS for the length of the launch shuts those out: with the full 64 x 64 filter bank the train step gets
    // 25 us slower, with the smaller banks of a pruned network 25 us faster - so only those take it here)
    return (PT_RES3 & 2) && res3_shape_ok(d) && (PT_RES3 & 4 || d->C * d->K <= kRes3BwdMaxBank) && aligned16(dy) &&
           aligned16(wt) && aligned16(dx) &&
           ((d->C % 8 == 0 && d->K % 8 == 0) || (d->flags & PT_CONV_PAD_ZERO));
}

// The first layer's own weight-gradient kernel takes image-like inputs: at most 4 channels at a pitch of 8, at most 64
// output channels, a filter of at most 8 x 8 at stride 1 or 2, and sizes whose byte offsets fit its 32-bit addressing.
inline bool stem_wgrad_ok(const pt_conv_desc* d) {
    return d->C <= 4 && d->x_cpitch == 8 && d->y_cpitch % 8 == 0 && d->K <= 64 && d->stride_h == d->stride_w &&
           d->stride_h >= 1 && d->stride_h <= 2 && d->R <= kStemMaxR && d->S <= 8 &&
           (int64_t)d->H * d->W * 16 <= 0x7fffffff && ((int64_t)2 * d->Q + 64) * d->y_cpitch * 2 <= 0x7fffffff &&
           (int64_t)d->N * ((d->P + 1) / 2) * ((d->Q + 63) / 64) <= 0x3fffffff;
}

inline StemWgradArgs make_stem_wgrad_args(const pt_conv_desc* d, const uint16_t* x, const uint16_t* dy, float* part) {
    StemWgradArgs s{};
    s.X = x; s.DY = dy; s.PART = part;
    s.N = d->N; s.H = d->H; s.W = d->W; s.P = d->P; s.Q = d->Q; s.K = d->K; s.KP = (int)round_up(d->K, 8);
    s.R = d->R; s.S = d->S; s.pad_h = d->pad_h; s.pad_w = d->pad_w; s.ypitch = d->y_cpitch;
    return s;
}

// one slab of [R][64][32] floats per workgroup of the launch
inline size_t stem_wgrad_ws(const pt_conv_desc* d) {
    StemWgradArgs s = make_stem_wgrad_args(d, nullptr, nullptr, nullptr);
    int slabs = 0;
    plan_stem_wgrad(s, &slabs);
    return (size_t)round_up((int64_t)(slabs > 0 ? slabs : 1) * d->R * kSwSlabRow * 4, 256);
}

inline size_t wgrad_ws(const pt_conv_desc* d) {
    const size_t a = plan_wgrad(d, true).ws_bytes, b = plan_wgrad(d, false).ws_bytes;
    const size_t c = stem_wgrad_ok(d) ? stem_wgrad_ws(d) : 0;
    return a > b ? (a > c ? a : c) : (b > c ? b : c);
}

// Workspace of the weight gradient with the regulariser folded into its reduction pass: at least one slab of partials
inline size_t wgrad_lasso_ws_of(const pt_conv_desc* d, const WgradPlan& p) {
    const size_t one = (size_t)round_up((int64_t)d->K * p.Mtot * 4, 256);
    return p.ws_bytes > one ? p.ws_bytes : one;
}

inline WgradArgs make_wgrad_args(const pt_conv_desc* d, const WgradPlan& p, const uint16_t* x, const uint16_t* dy,
                                 float* dw, void* ws) {
    WgradArgs a{};
    a.X = x; a.DY = dy;
    a.pixels = d->N * d->P * d->Q;
    a.Q = make_fastdiv((uint32_t)d->Q); a.P = make_fastdiv((uint32_t)d->P);
    a.H = d->H; a.W = d->W; a.xpitch = d->x_cpitch; a.ypitch = d->y_cpitch;
    a.stride_h = d->stride_h; a.stride_w = d->stride_w; a.pad_h = d->pad_h; a.pad_w = d->pad_w;
    a.S = d->S; a.RS = d->R * d->S; a.C = d->C; a.CP = p.CP; a.KP = p.KP; a.Mtot = p.Mtot; a.K = d->K;
    a.tiles_n = p.tiles_n; a.tiles_m = p.tiles_m; a.tiles_per_tap = p.tiles_per_tap; a.fold = p.fold;
    a.iters_total = p.iters_total; a.iters_per_split = p.iters_per_split; a.splits = p.splits;
    a.affine = d->stride_h == 1 && d->stride_w == 1 && d->P == d->H && d->Q == d->W;
    a.x_all_valid = a.affine && d->R == 1 && d->S == 1 && d->pad_h == 0 && d->pad_w == 0;
    a.wpitch = d->w_cpitch;
    a.direct = p.splits == 1;
    a.OUT = a.direct ? dw : (float*)ws;
    a.out_row_pitch = p.Mtot;
    a.o_vec = (d->w_cpitch % 4 == 0) && aligned16(dw);
    return a;
}

inline hipError_t launch_wgrad(WgradArgs& a, const WgradPlan& p, bool vec, hipStream_t st) {
    if (!p.dl) {
        if (!vec) return launch_wgrad_cfg<kWgBM, kWgBN, kWgBK, 2, 2, 2, false>(a, st);
        return launch_wgrad_cfg<kWgBM, kWgBN, kWgBK, 2, 2, 2>(a, st);
    }
    // wave grids and pipeline depths from measurements on ResNet-50 shapes
    // 128 x 128: eight waves of 32 x 64 outputs, no wave groups (with 32-pixel steps a group would get one sub-step per
    // stage and nothing to read ahead): 6 % faster alone than two groups of 2 x 2 waves, 0.4 % in the step
    if (p.BM == 128 && p.BN == 128) return launch_wgrad_dl_cfg<128, 128, kWgDlBKPBig, 4, 2, 5, 1>(a, st);
    if (p.BM == 64 && p.BN == 128) return launch_wgrad_dl_cfg<64, 128, kWgDlBKP, 2, 2, 3, 2>(a, st);
    if (p.BM == 128 && p.BN == 64) return launch_wgrad_dl_cfg<128, 64, kWgDlBKP, 2, 2, 3, 2>(a, st);
    return launch_wgrad_dl_cfg<64, 64, kWgDlBKP, 2, 2, 4, 2>(a, st);
}

}  // namespace pt
