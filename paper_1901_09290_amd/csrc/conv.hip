// Implicit-GEMM convolution kernels for gfx950: forward, input gradient, weight gradient
// (Sec. 2.1, Alg. 1 ForwardProp/BackProp, Eq. 4).  bf16 operands, fp32 accumulation on the
// 32x32x16 bf16 MFMA, NHWC activations, KRSC weights.
//
// forward / input gradient share one kernel (k_igemm): output pixels x output channels, reduced over
// (filter tap, reduction channel).  Both operands are contiguous along the reduction channel, which
// is what the MFMA wants per lane (8 consecutive k), so 16-byte global loads go to LDS unchanged.
//   forward:        A = x gathered at (p*stride - pad + r, q*stride - pad + s),  B = w[k][r][s][c]
//   input gradient: per stride-parity class of input pixels (dense sub-problem with only the taps
//                   that can reach that class), A = dy gathered at (h' + off - jr, w' + off - js),
//                   B = w transposed to [c][r][s][k] in the workspace.
// The MFMA "row" operand is the weight tile and the "column" operand the pixel tile, so each lane's
// four consecutive accumulator rows are four consecutive output channels of one pixel (one 8-byte
// store of bf16).
//
// weight gradient (k_wgrad): output (tap, c) x k, reduced over output pixels.  Memory is contiguous
// along channels, not along the reduction axis, so tiles are stored pixel-major in LDS exactly as
// loaded and read back with the LDS transpose read (ds_read_b64_tr_b16), which hands every lane four
// consecutive reduction elements of one channel.  The pixel range is split over workgroups; partial
// sums go to an fp32 workspace and are combined in a fixed order by k_wgrad_reduce.
//
// Ragged channel counts: the reduction axis is laid out as taps x (C rounded up to 8), so a ragged C
// costs one partially filled 8-vector per tap; lanes beyond C are masked to zero on load.  32-wide
// accumulator blocks that lie wholly outside the logical output are skipped.
#include "conv_kernels.h"

namespace pt {

// w[K][RS][wpitch] -> wt[C][RS][kpitch]  (bf16), for the input-gradient GEMM.
__global__ void k_transpose_w(const uint16_t* __restrict__ w, int K, int RS, int C, int wpitch,
                              uint16_t* __restrict__ wt, int kpitch) {
    __shared__ uint16_t tile[32][33];
    const int rs = blockIdx.z;
    const int k0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int i = ty; i < 32; i += 8) {
        const int k = k0 + i, c = c0 + tx;
        tile[i][tx] = (k < K && c < C) ? w[((int64_t)k * RS + rs) * wpitch + c] : (uint16_t)0;
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int c = c0 + i, k = k0 + tx;
        if (c < C && k < kpitch) wt[((int64_t)c * RS + rs) * kpitch + k] = tile[tx][i];
    }
}

// The same transposition for many layers in one launch (descriptors in the kernel arguments).
constexpr int kMaxTransposeJobs = 64;
struct TransposeJob {
    const uint16_t* w;
    uint16_t* wt;
    int K, RS, C, wpitch, kpitch, blk0, nbx, nby;
};
struct TransposeJobs {
    TransposeJob j[kMaxTransposeJobs];
    int n;
};
__global__ __launch_bounds__(256) void k_transpose_w_multi(const TransposeJobs jobs) {
    __shared__ uint16_t tile[32][33];
    int lo = 0, hi = jobs.n - 1;  // last job whose blk0 <= blockIdx.x
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs.j[mid].blk0 <= (int)blockIdx.x) lo = mid;
        else hi = mid - 1;
    }
    const TransposeJob& jb = jobs.j[lo];
    int b = blockIdx.x - jb.blk0;
    const int bx = b % jb.nbx;
    b /= jb.nbx;
    const int by = b % jb.nby, rs = b / jb.nby;
    const int k0 = by * 32, c0 = bx * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int i = ty; i < 32; i += 8) {
        const int k = k0 + i, c = c0 + tx;
        tile[i][tx] = (k < jb.K && c < jb.C) ? jb.w[((int64_t)k * jb.RS + rs) * jb.wpitch + c] : (uint16_t)0;
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int c = c0 + i, k = k0 + tx;
        if (c < jb.C && k < jb.kpitch) jb.wt[((int64_t)c * jb.RS + rs) * jb.kpitch + k] = tile[tx][i];
    }
}

// Zero the destination pixels of a stride-parity class that no output pixel reaches.  One thread clears
// 8 channels (one 16-byte store when the rows are 16-byte aligned).
__global__ void k_zero_class(uint16_t* __restrict__ D, int64_t pixels, int gH, int gW, int DH, int DW, int d_hmul,
                             int d_hadd, int d_wmul, int d_wadd, int dpitch, int Nout, int vec16) {
    const int cv = (Nout + 7) >> 3;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= pixels * cv) return;
    const int64_t m = t / cv;
    const int ch = (int)(t - m * cv) * 8;
    const int gHW = gH * gW;
    const int64_t n = m / gHW;
    const int rem = (int)(m - n * gHW);
    const int gi = rem / gW, gj = rem - gi * gW;
    uint16_t* dst = D + ((n * DH + gi * d_hmul + d_hadd) * DW + gj * d_wmul + d_wadd) * dpitch + ch;
    if (vec16 && ch + 7 < Nout) {
        *reinterpret_cast<uint4*>(dst) = make_uint4(0u, 0u, 0u, 0u);
    } else {
        for (int e = 0; e < 8; ++e)
            if (ch + e < Nout) dst[e] = 0;
    }
}

// dw[k][tap][c] = sum over splits of partial[split][k][tap*CP + c], in a fixed order: a workgroup owns
// 64 consecutive outputs; wavefront v adds the splits v, v+8, v+16, ... (four loads in flight), and the
// eight wavefront sums are added in ascending order.  Results do not depend on timing.
// LASSO: the gradient of the group-lasso penalty (Eq. 1-2) is added on the way out, with the arithmetic of
// k_group_lasso_grad: dw = sum + lambda * (w * (1/out_norm[k] + 1/in_norm[c])), a zero norm contributing 0.
constexpr int kReduceWaves = 8;
constexpr int kReduceWideMaxSplits = 16;
constexpr int64_t kReduceWideMinOutputs = 64 * 1024;
struct ReduceLasso {
    const float* w;         // [K][RS][wpitch], the pitch of dw
    const float* out_norm;  // [K]
    const float* in_norm;   // [C]
    float lambda;
    uint32_t flags;         // PT_LASSO_OUT | PT_LASSO_IN
};
template <bool LASSO>
__global__ __launch_bounds__(64 * kReduceWaves) void k_wgrad_reduce(const float* __restrict__ part, int splits, int K,
                                                                     int RS, int C, int CP, int wpitch,
                                                                     float* __restrict__ dw, const ReduceLasso rl) {
    __shared__ float red[kReduceWaves][64];
    const int Mtot = RS * CP;
    const int64_t total = (int64_t)K * Mtot;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t t = (int64_t)blockIdx.x * 64 + lane;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (t < total) {
        int i = wave;
        for (; i + 3 * kReduceWaves < splits; i += 4 * kReduceWaves) {
            s0 += part[(int64_t)i * total + t];
            s1 += part[(int64_t)(i + kReduceWaves) * total + t];
            s2 += part[(int64_t)(i + 2 * kReduceWaves) * total + t];
            s3 += part[(int64_t)(i + 3 * kReduceWaves) * total + t];
        }
        for (; i < splits; i += kReduceWaves) s0 += part[(int64_t)i * total + t];
    }
    red[wave][lane] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (wave == 0 && t < total) {
        float s = 0.f;
#pragma unroll
        for (int v = 0; v < kReduceWaves; ++v) s += red[v][lane];
        const int64_t k = t / Mtot;
        const int mrow = (int)(t - k * Mtot);
        const int tp = mrow / CP, c = mrow - tp * CP;
        if (c < C) {
            const int64_t o = (k * RS + tp) * wpitch + c;
            if constexpr (LASSO) {
                const float on = (rl.flags & PT_LASSO_OUT) ? rl.out_norm[k] : 0.f;
                const float in = (rl.flags & PT_LASSO_IN) ? rl.in_norm[c] : 0.f;
                const float inv_out = on > 0.f ? 1.0f / on : 0.f, inv_in = in > 0.f ? 1.0f / in : 0.f;
                s += rl.lambda * (rl.w[o] * (inv_out + inv_in));
            }
            dw[o] = s;
        }
    }
}

// The same sum for launches with few splits and many outputs: one thread per four consecutive outputs of the slab
// (16-byte loads, the splits added in ascending order with four loads in flight), so a workgroup covers 1024 outputs
// instead of 64.  CP is a multiple of 8: the four outputs share a filter tap.
template <bool LASSO>
__global__ __launch_bounds__(256) void k_wgrad_reduce4(const float* __restrict__ part, int splits, int K, int RS, int C,
                                                       int CP, int wpitch, int o_vec, float* __restrict__ dw,
                                                       const ReduceLasso rl) {
    const int Mtot = RS * CP;
    const int64_t total = (int64_t)K * Mtot;
    const int64_t t = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (t >= total) return;
    const int64_t k = t / Mtot;
    const int mrow = (int)(t - k * Mtot);
    const int tp = mrow / CP, c = mrow - tp * CP;
    if (c >= C) return;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    int i = 0;
    for (; i + 3 < splits; i += 4) {
        const float4 a0 = *reinterpret_cast<const float4*>(part + (int64_t)i * total + t);
        const float4 a1 = *reinterpret_cast<const float4*>(part + (int64_t)(i + 1) * total + t);
        const float4 a2 = *reinterpret_cast<const float4*>(part + (int64_t)(i + 2) * total + t);
        const float4 a3 = *reinterpret_cast<const float4*>(part + (int64_t)(i + 3) * total + t);
        s.x = (((s.x + a0.x) + a1.x) + a2.x) + a3.x;
        s.y = (((s.y + a0.y) + a1.y) + a2.y) + a3.y;
        s.z = (((s.z + a0.z) + a1.z) + a2.z) + a3.z;
        s.w = (((s.w + a0.w) + a1.w) + a2.w) + a3.w;
    }
    for (; i < splits; ++i) {
        const float4 a0 = *reinterpret_cast<const float4*>(part + (int64_t)i * total + t);
        s.x += a0.x; s.y += a0.y; s.z += a0.z; s.w += a0.w;
    }
    const int64_t o = (k * RS + tp) * wpitch + c;
    float v[4] = {s.x, s.y, s.z, s.w};
    const bool whole = o_vec && c + 3 < C;
    if constexpr (LASSO) {
        const float on = (rl.flags & PT_LASSO_OUT) ? rl.out_norm[k] : 0.f;
        const float inv_out = on > 0.f ? 1.0f / on : 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (c + e < C) {
                const float in = (rl.flags & PT_LASSO_IN) ? rl.in_norm[c + e] : 0.f;
                v[e] += rl.lambda * (rl.w[o + e] * (inv_out + (in > 0.f ? 1.0f / in : 0.f)));
            }
        }
    }
    if (whole) {
        *reinterpret_cast<float4*>(dw + o) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (c + e < C) dw[o + e] = v[e];
    }
}

// The same for the slabs of k_stem_wgrad, [slab][r][64 output channels][8 taps x 4 channels]: one output per lane, the
// slabs spread over eight wavefronts (four loads in flight each) and the eight sums added in ascending order.
template <bool LASSO>
__global__ __launch_bounds__(64 * kReduceWaves) void k_stem_wgrad_reduce(const float* __restrict__ part, int slabs, int K,
                                                                          int R, int S, int C, int wpitch,
                                                                          float* __restrict__ dw, const ReduceLasso rl) {
    __shared__ float red[kReduceWaves][64];
    const int64_t total = (int64_t)R * kSwSlabRow;  // a multiple of 64
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blockIdx.x * 64 + lane;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int i = wave;
    for (; i + 3 * kReduceWaves < slabs; i += 4 * kReduceWaves) {
        s0 += part[(int64_t)i * total + t];
        s1 += part[(int64_t)(i + kReduceWaves) * total + t];
        s2 += part[(int64_t)(i + 2 * kReduceWaves) * total + t];
        s3 += part[(int64_t)(i + 3 * kReduceWaves) * total + t];
    }
    for (; i < slabs; i += kReduceWaves) s0 += part[(int64_t)i * total + t];
    red[wave][lane] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (wave == 0) {
        float s = 0.f;
#pragma unroll
        for (int v = 0; v < kReduceWaves; ++v) s += red[v][lane];
        const int n = t & 31, k = (t >> 5) & 63, r = t >> 11;
        const int fs = n >> 2, c = n & 3;
        if (k < K && fs < S && c < C) {
            const int64_t o = ((int64_t)(k * R + r) * S + fs) * wpitch + c;
            if constexpr (LASSO) {
                const float on = (rl.flags & PT_LASSO_OUT) ? rl.out_norm[k] : 0.f;
                const float in = (rl.flags & PT_LASSO_IN) ? rl.in_norm[c] : 0.f;
                const float inv_out = on > 0.f ? 1.0f / on : 0.f, inv_in = in > 0.f ? 1.0f / in : 0.f;
                s += rl.lambda * (rl.w[o] * (inv_out + inv_in));
            }
            dw[o] = s;
        }
    }
}

}  // namespace pt

#include "conv_host.h"

using namespace pt;

extern "C" int32_t pt_conv_fwd_workspace_bytes(const pt_conv_desc* d, size_t* bytes) {
    if (!bytes) return PT_ERR_NULL;
    int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    *bytes = 0;
    return PT_OK;
}

extern "C" int32_t pt_conv_bwd_data_workspace_bytes(const pt_conv_desc* d, size_t* bytes) {
    if (!bytes) return PT_ERR_NULL;
    int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    *bytes = bwd_data_ws(d);
    return PT_OK;
}

extern "C" int32_t pt_conv_bwd_weight_workspace_bytes(const pt_conv_desc* d, size_t* bytes) {
    if (!bytes) return PT_ERR_NULL;
    int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    *bytes = wgrad_ws(d);
    return PT_OK;
}

static int32_t hip_status(hipError_t e) {
    if (e != hipSuccess) {
        set_hip_error(e);
        return PT_ERR_LAUNCH;
    }
    return launch_status();
}

// image-like first layer (at most 4 channels at a pitch of 8, zero padding vouched for): its own kernel
static bool stem_fwd_ok(const pt_conv_desc* d, const uint16_t* x, const uint16_t* w, const uint16_t* y) {
    return d->C <= 4 && d->x_cpitch == 8 && d->w_cpitch == 8 && (d->flags & PT_CONV_PAD_ZERO) && d->y_cpitch % 8 == 0 &&
           aligned16(x) && aligned16(w) && aligned16(y) && d->stride_h == d->stride_w && d->stride_h <= 2 &&
           d->R <= kStemMaxR && d->S <= 8 && (int64_t)d->H * d->W * 16 <= 0x7fffffff;
}

extern "C" int32_t pt_conv_fwd(const pt_conv_desc* d, const uint16_t* x, const uint16_t* w, uint16_t* y, void* ws,
                               size_t ws_bytes, void* stream) {
    (void)ws;
    (void)ws_bytes;
    int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    if (!x || !w || !y) return PT_ERR_NULL;
    if (stem_fwd_ok(d, x, w, y)) {
        StemArgs s{x, w, y, d->N, d->H, d->W, d->P, d->Q, d->K, d->R, d->S, d->pad_h, d->pad_w, d->y_cpitch, 0, 0, 0, 0};
        return hip_status(launch_stem_fwd(s, d->stride_h, kStemSlots, (hipStream_t)stream));
    }
    if (res3_fwd_ok(d, x, w, y)) {  // early 3 x 3 layer: the filter bank stays in LDS
        const int cinp = (int)round_up(d->C, 8);
        Res3Args r{x, w, y, d->N, d->H, d->W, d->C, cinp, d->x_cpitch, d->K, d->w_cpitch, d->y_cpitch, 0, 0, 0, 0, 0};
        return hip_status(launch_conv3x3_res(r, false, (hipStream_t)stream));
    }
    IgemmArgs a = make_fwd_args(d, x, w, y);
    const bool vec = d->x_cpitch % 8 == 0 && d->w_cpitch % 8 == 0 && aligned16(x) && aligned16(w);
    return hip_status(launch_igemm(a, vec, (hipStream_t)stream));
}

extern "C" int32_t pt_conv_fwd_batched(const pt_conv_desc* descs, const uint16_t* const* x, const uint16_t* const* w,
                                       uint16_t* const* y, int32_t n, void* stream) {
    if (n <= 0) return PT_ERR_SHAPE;
    if (!descs || !x || !w || !y) return PT_ERR_NULL;
    for (int i = 0; i < n; ++i) {
        const int32_t rc = check_desc(&descs[i]);
        if (rc != PT_OK) return rc;
        if (!x[i] || !w[i] || !y[i]) return PT_ERR_NULL;
    }
    hipStream_t st = (hipStream_t)stream;
    IgemmArgs pend_a[kIgemmMaxProblems];
    IgemmDlPlan pend_p[kIgemmMaxProblems];
    int n_pend = 0;
    auto flush = [&]() -> int32_t {
        if (n_pend == 0) return PT_OK;
        const int32_t r = hip_status(launch_igemm_dl_planned(pend_a, pend_p, n_pend, st));
        n_pend = 0;
        return r;
    };
    for (int i = 0; i < n; ++i) {
        const pt_conv_desc* d = &descs[i];
        if (stem_fwd_ok(d, x[i], w[i], y[i]) || res3_fwd_ok(d, x[i], w[i], y[i])) {  // layers with a kernel of their own
            const int32_t rc = pt_conv_fwd(d, x[i], w[i], y[i], nullptr, 0, stream);
            if (rc != PT_OK) return rc;
            continue;
        }
        IgemmArgs a = make_fwd_args(d, x[i], w[i], y[i]);
        const bool vec = d->x_cpitch % 8 == 0 && d->w_cpitch % 8 == 0 && aligned16(x[i]) && aligned16(w[i]);
        bool planned = false;
        int32_t rc = hip_status(launch_igemm(a, vec, st, &pend_p[n_pend], &planned));
        if (rc == PT_OK && planned) {
            pend_a[n_pend++] = a;
            if (n_pend == kIgemmMaxProblems) rc = flush();
        }
        if (rc != PT_OK) return rc;
    }
    return flush();
}

// Input gradient from weights already in [C][RS][round_up(K,8)] order: one implicit GEMM per stride-parity class.
static int32_t bwd_data_classes(const pt_conv_desc* d, const uint16_t* dy, const uint16_t* wt, uint16_t* dx,
                                hipStream_t st) {
    int32_t rc = PT_OK;
    if (res3_bwd_ok(d, dy, wt, dx)) {  // the same kernel on dy with the k-innermost filter copy and mirrored taps
        const int kp = (int)round_up(d->K, 8);
        Res3Args r{dy, wt, dx, d->N, d->H, d->W, d->K, kp, d->y_cpitch, d->C, kp, d->x_cpitch, 0, 0, 0, 0, 0};
        return hip_status(launch_conv3x3_res(r, true, st));
    }
    // A filter no larger than the stride reaches only some stride-parity classes of input pixels.  When class
    // (0, 0) is the only one with taps, its launch also clears the other classes (they tile into cells anchored at
    // its pixels), which saves up to stride_h * stride_w - 1 small launches; this needs the vector store path and a
    // channel count whose last 8-chunk may be written whole.
    int with_taps = 0;
    for (int ca = 0; ca < d->stride_h; ++ca)
        for (int cb = 0; cb < d->stride_w; ++cb) {
            const BwdClass c = bwd_data_class(d, ca, cb);
            if (c.gH > 0 && c.gW > 0 && c.TR > 0 && c.TS > 0) ++with_taps;
        }
    const BwdClass c00 = bwd_data_class(d, 0, 0);
    const bool vec_all = d->x_cpitch % 8 == 0 && d->y_cpitch % 8 == 0 && aligned16(dx) && aligned16(dy);
    const bool fuse_zero = with_taps == 1 && c00.TR > 0 && c00.TS > 0 && d->stride_h * d->stride_w > 1 && vec_all &&
                           (d->C % 8 == 0 || (d->flags & PT_CONV_PAD_ZERO)) && c00.TR * c00.TS <= 64;
    // Classes that the direct kernel takes are collected and sent out together: those that chose the same instantiation
    // share a launch (a 3 x 3 filter at stride 2 has four classes of 1, 2, 2 and 4 taps: four short launches one after
    // the other otherwise).
    IgemmArgs pend_a[kIgemmMaxProblems];
    IgemmDlPlan pend_p[kIgemmMaxProblems];
    int n_pend = 0;
    auto flush = [&]() -> int32_t {
        if (n_pend == 0) return PT_OK;
        const int32_t r = hip_status(launch_igemm_dl_planned(pend_a, pend_p, n_pend, st));
        n_pend = 0;
        return r;
    };
    for (int ca = 0; ca < d->stride_h; ++ca) {
        for (int cb = 0; cb < d->stride_w; ++cb) {
            BwdClass c = bwd_data_class(d, ca, cb);
            if (c.gH == 0 || c.gW == 0) continue;
            if (fuse_zero && (ca != 0 || cb != 0)) continue;  // cleared by the launch of class (0, 0)
            if (c.TR == 0 || c.TS == 0) {
                const int64_t pixels = (int64_t)d->N * c.gH * c.gW;
                const int64_t nblk = ceil_div(pixels * ceil_div(d->C, 8), 256);
                if (nblk > 0x7fffffff) return PT_ERR_UNSUPPORTED;
                const int vec16 = (d->x_cpitch % 8 == 0) && aligned16(dx);
                hipLaunchKernelGGL(k_zero_class, dim3((unsigned)nblk), dim3(256), 0, st, dx, pixels, c.gH, c.gW, d->H, d->W,
                                   d->stride_h, ca, d->stride_w, cb, d->x_cpitch, d->C, vec16);
                rc = launch_status();
            } else {
                IgemmArgs a = make_bwd_data_args(d, c, ca, cb, dy, wt, dx);
                if (fuse_zero) {
                    a.zf_h = d->stride_h;
                    a.zf_w = d->stride_w;
                }
                bool planned = false;
                rc = hip_status(launch_igemm(a, d->y_cpitch % 8 == 0 && aligned16(dy), st, &pend_p[n_pend], &planned));
                if (rc == PT_OK && planned) {
                    pend_a[n_pend++] = a;
                    if (n_pend == kIgemmMaxProblems) rc = flush();
                }
            }
            if (rc != PT_OK) return rc;
        }
    }
    return flush();
}

// Forward convolution with the statistics epilogue: only the direct kernel has it.
static int32_t fwd_stats_supported(const pt_conv_desc* d, const uint16_t* x, const uint16_t* w, const uint16_t* y) {
    const bool vec = d->x_cpitch % 8 == 0 && d->w_cpitch % 8 == 0 && d->y_cpitch % 8 == 0 && aligned16(x) && aligned16(w) &&
                     aligned16(y);
    if (!vec || d->R * d->S > 64) return PT_ERR_UNSUPPORTED;
    if (d->C % 8 != 0 && !(d->flags & PT_CONV_PAD_ZERO)) return PT_ERR_UNSUPPORTED;
    return PT_OK;
}

extern "C" int32_t pt_conv_fwd_stats_workspace_bytes(const pt_conv_desc* d, size_t* bytes, int32_t* n_partial) {
    const int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    if (!bytes || !n_partial) return PT_ERR_NULL;
    *n_partial = (int32_t)ceil_div((int64_t)d->N * d->P * d->Q, 128);
    *bytes = (size_t)round_up((int64_t)2 * *n_partial * d->K * 4, 256);
    return PT_OK;
}

extern "C" int32_t pt_conv_fwd_stats(const pt_conv_desc* d, const uint16_t* x, const uint16_t* w, uint16_t* y, float* sums,
                                     size_t sums_bytes, void* stream) {
    int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    if (!x || !w || !y || !sums) return PT_ERR_NULL;
    rc = fwd_stats_supported(d, x, w, y);
    if (rc != PT_OK) return rc;
    const int64_t n_partial = ceil_div((int64_t)d->N * d->P * d->Q, 128);
    if (sums_bytes < (size_t)(2 * n_partial * d->K * 4)) return PT_ERR_WORKSPACE;
    IgemmArgs a = make_fwd_args(d, x, w, y);
    a.stats = sums;
    return hip_status(launch_igemm(a, true, (hipStream_t)stream));
}

extern "C" int32_t pt_conv_bwd_data(const pt_conv_desc* d, const uint16_t* dy, const uint16_t* w, uint16_t* dx,
                                    void* ws, size_t ws_bytes, void* stream) {
    int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    if (!dy || !w || !dx || !ws) return PT_ERR_NULL;
    if (ws_bytes < bwd_data_ws(d)) return PT_ERR_WORKSPACE;
    if (!aligned16(ws)) return PT_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    const int RS = d->R * d->S;
    const int kpitch = (int)round_up(d->K, 8);
    uint16_t* wt = (uint16_t*)ws;
    hipLaunchKernelGGL(k_transpose_w, dim3((unsigned)ceil_div(d->C, 32), (unsigned)ceil_div(kpitch, 32), RS), dim3(256),
                       0, st, w, d->K, RS, d->C, d->w_cpitch, wt, kpitch);
    rc = launch_status();
    if (rc != PT_OK) return rc;
    return bwd_data_classes(d, dy, wt, dx, st);
}

extern "C" int32_t pt_conv_bwd_data_crsk(const pt_conv_desc* d, const uint16_t* dy, const uint16_t* wt, uint16_t* dx,
                                         void* stream) {
    int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    if (!dy || !wt || !dx) return PT_ERR_NULL;
    if (!aligned16(wt)) return PT_ERR_SHAPE;
    return bwd_data_classes(d, dy, wt, dx, (hipStream_t)stream);
}

extern "C" int32_t pt_weights_to_crsk_batched(const pt_layer_crsk* layers, int32_t n, void* stream) {
    if (n < 0) return PT_ERR_SHAPE;
    if (n == 0) return PT_OK;
    if (!layers) return PT_ERR_NULL;
    for (int i = 0; i < n; ++i) {
        const pt_layer_crsk& l = layers[i];
        if (!l.w || !l.wt) return PT_ERR_NULL;
        if (l.K <= 0 || l.RS <= 0 || l.C <= 0 || l.w_cpitch < l.C) return PT_ERR_SHAPE;
        if ((int64_t)ceil_div(l.C, 32) * ceil_div(round_up(l.K, 8), 32) * l.RS > 0x3fffffff) return PT_ERR_UNSUPPORTED;
    }
    TransposeJobs t;
    t.n = 0;
    int64_t blocks = 0;
    auto flush = [&]() -> int32_t {
        if (t.n == 0) return PT_OK;
        hipLaunchKernelGGL(k_transpose_w_multi, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, t);
        t.n = 0;
        blocks = 0;
        return launch_status();
    };
    for (int i = 0; i < n; ++i) {
        const pt_layer_crsk& l = layers[i];
        const int kpitch = (int)round_up(l.K, 8);
        const int nbx = (int)ceil_div(l.C, 32), nby = (int)ceil_div(kpitch, 32);
        const int64_t nb = (int64_t)nbx * nby * l.RS;
        if (blocks + nb > 0x3fffffff) {
            const int32_t rc = flush();
            if (rc != PT_OK) return rc;
        }
        t.j[t.n++] = TransposeJob{l.w, l.wt, l.K, l.RS, l.C, l.w_cpitch, kpitch, (int)blocks, nbx, nby};
        blocks += nb;
        if (t.n == kMaxTransposeJobs) {
            const int32_t rc = flush();
            if (rc != PT_OK) return rc;
        }
    }
    return flush();
}

// Few slices over many outputs take the four-outputs-per-thread reduction, the rest the one-output-per-lane form.
static bool reduce_is_wide(const pt_conv_desc* d, const WgradPlan& p) {
    const int64_t work = (int64_t)d->K * p.Mtot;
    return p.splits <= kReduceWideMaxSplits && work >= kReduceWideMinOutputs && p.Mtot % 4 == 0;
}

extern "C" int32_t pt_conv_bwd_weight_plan(const pt_conv_desc* d, int32_t aligned, pt_wgrad_plan_info* info) {
    if (!info) return PT_ERR_NULL;
    const int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    const bool vec = aligned != 0 && d->x_cpitch % 8 == 0 && d->y_cpitch % 8 == 0;
    if (vec && stem_wgrad_ok(d)) {  // the first layer's own kernel: one slab per workgroup, always reduced
        StemWgradArgs s = make_stem_wgrad_args(d, nullptr, nullptr, nullptr);
        int slabs = 0;
        plan_stem_wgrad(s, &slabs);
        info->splits = slabs;
        info->tiles = 1;
        info->reduce_kind = PT_WGRAD_REDUCE_DEEP;
        info->tile_m = 32;
        info->tile_n = 64;
        return PT_OK;
    }
    const WgradPlan p = plan_wgrad(d, vec);
    info->splits = p.splits;
    info->tiles = p.tiles_m * p.tiles_n;
    info->reduce_kind = p.splits == 1 ? PT_WGRAD_REDUCE_NONE : (reduce_is_wide(d, p) ? PT_WGRAD_REDUCE_WIDE : PT_WGRAD_REDUCE_DEEP);
    info->tile_m = p.BM;
    info->tile_n = p.BN;
    return PT_OK;
}

// rl == nullptr: plain weight gradient.  Otherwise the regulariser's gradient is added where dw is written: in the
// reduction pass of a split launch, in the epilogue of an unsplit launch of the direct kernel, and for an unsplit
// launch of the register-staged kernel in a reduction pass over one slab of partial sums.
static int32_t bwd_weight_impl(const pt_conv_desc* d, const uint16_t* x, const uint16_t* dy, float* dw, void* ws,
                               size_t ws_bytes, void* stream, const ReduceLasso* rl) {
    int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    if (!x || !dy || !dw) return PT_ERR_NULL;
    // the direct kernel needs 16-byte aligned rows; it keeps one tile row block per filter tap
    const bool vec = d->x_cpitch % 8 == 0 && d->y_cpitch % 8 == 0 && aligned16(x) && aligned16(dy);
    hipStream_t st = (hipStream_t)stream;
    if (vec && stem_wgrad_ok(d)) {  // image-like first layer: its own kernel, one slab of partial sums per workgroup
        const size_t need = stem_wgrad_ws(d);
        if (!ws) return PT_ERR_NULL;
        if (ws_bytes < need) return PT_ERR_WORKSPACE;
        if (!aligned16(ws)) return PT_ERR_SHAPE;
        StemWgradArgs s = make_stem_wgrad_args(d, x, dy, (float*)ws);
        int slabs = 0;
        plan_stem_wgrad(s, &slabs);
        if (slabs <= 0) return PT_OK;
        rc = hip_status(launch_stem_wgrad(s, slabs, d->stride_h, st));
        if (rc != PT_OK) return rc;
        const ReduceLasso none{};
        const unsigned nb = (unsigned)(d->R * (kSwSlabRow / 64));
        if (rl)
            hipLaunchKernelGGL(k_stem_wgrad_reduce<true>, dim3(nb), dim3(64 * kReduceWaves), 0, st, (const float*)ws, slabs, d->K,
                               d->R, d->S, d->C, d->w_cpitch, dw, *rl);
        else
            hipLaunchKernelGGL(k_stem_wgrad_reduce<false>, dim3(nb), dim3(64 * kReduceWaves), 0, st, (const float*)ws, slabs, d->K,
                               d->R, d->S, d->C, d->w_cpitch, dw, none);
        return launch_status();
    }
    const WgradPlan p = plan_wgrad(d, vec);
    const size_t need = rl ? wgrad_lasso_ws_of(d, p) : p.ws_bytes;
    if (need > 0 && !ws) return PT_ERR_NULL;
    if (ws_bytes < need) return PT_ERR_WORKSPACE;
    if (need > 0 && !aligned16(ws)) return PT_ERR_SHAPE;
    WgradArgs a = make_wgrad_args(d, p, x, dy, dw, ws);
    if (rl && a.direct && p.dl && aligned16(rl->w)) {  // the direct kernel's own epilogue adds the term (vector loads of w)
        a.lw = rl->w;
        a.l_on = (rl->flags & PT_LASSO_OUT) ? rl->out_norm : nullptr;
        a.l_in = (rl->flags & PT_LASSO_IN) ? rl->in_norm : nullptr;
        a.l_lambda = rl->lambda;
    } else if (rl) {               // the reduction pass adds it (one slab when the launch is not split)
        a.direct = 0;
        a.OUT = (float*)ws;
    }
    rc = hip_status(launch_wgrad(a, p, vec, st));
    if (rc != PT_OK) return rc;
    if (!a.direct) {
        const int64_t work = (int64_t)d->K * p.Mtot;
        const int64_t nblk = ceil_div(work, 64);
        if (nblk > 0x7fffffff) return PT_ERR_UNSUPPORTED;
        // few splits over many outputs: the four-outputs-per-thread form; many splits over few outputs: one output per
        // lane with the splits spread over eight wavefronts
        const bool wide = reduce_is_wide(d, p);
        const ReduceLasso none{};
        if (wide) {
            const unsigned nb4 = (unsigned)ceil_div(work / 4, 256);
            if (rl)
                hipLaunchKernelGGL(k_wgrad_reduce4<true>, dim3(nb4), dim3(256), 0, st, (const float*)ws, p.splits, d->K, a.RS,
                                   d->C, p.CP, d->w_cpitch, a.o_vec, dw, *rl);
            else
                hipLaunchKernelGGL(k_wgrad_reduce4<false>, dim3(nb4), dim3(256), 0, st, (const float*)ws, p.splits, d->K, a.RS,
                                   d->C, p.CP, d->w_cpitch, a.o_vec, dw, none);
        } else if (rl) {
            hipLaunchKernelGGL(k_wgrad_reduce<true>, dim3((unsigned)nblk), dim3(64 * kReduceWaves), 0, st, (const float*)ws,
                               p.splits, d->K, a.RS, d->C, p.CP, d->w_cpitch, dw, *rl);
        } else {
            hipLaunchKernelGGL(k_wgrad_reduce<false>, dim3((unsigned)nblk), dim3(64 * kReduceWaves), 0, st, (const float*)ws,
                               p.splits, d->K, a.RS, d->C, p.CP, d->w_cpitch, dw, none);
        }
        rc = launch_status();
    }
    return rc;
}

extern "C" int32_t pt_conv_bwd_weight(const pt_conv_desc* d, const uint16_t* x, const uint16_t* dy, float* dw, void* ws,
                                      size_t ws_bytes, void* stream) {
    return bwd_weight_impl(d, x, dy, dw, ws, ws_bytes, stream, nullptr);
}

extern "C" int32_t pt_conv_bwd_weight_lasso_workspace_bytes(const pt_conv_desc* d, size_t* bytes) {
    if (!bytes) return PT_ERR_NULL;
    int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    const size_t a = wgrad_lasso_ws_of(d, plan_wgrad(d, true)), b = wgrad_lasso_ws_of(d, plan_wgrad(d, false));
    const size_t c = stem_wgrad_ok(d) ? stem_wgrad_ws(d) : 0;
    *bytes = a > b ? (a > c ? a : c) : (b > c ? b : c);
    return PT_OK;
}

extern "C" int32_t pt_conv_bwd_weight_lasso(const pt_conv_desc* d, const uint16_t* x, const uint16_t* dy, const float* w,
                                            const float* out_norm, const float* in_norm, float lambda, uint32_t flags,
                                            float* dw, void* ws, size_t ws_bytes, void* stream) {
    if (!w || !out_norm || !in_norm) return PT_ERR_NULL;
    if (flags & ~(PT_LASSO_OUT | PT_LASSO_IN)) return PT_ERR_UNSUPPORTED;
    const ReduceLasso rl{w, out_norm, in_norm, lambda, flags};
    return bwd_weight_impl(d, x, dy, dw, ws, ws_bytes, stream, &rl);
}
