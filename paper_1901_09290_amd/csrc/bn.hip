// Feature (batch) normalisation over the N*H*W pixels of an NHWC bf16 tensor, training mode: forward and
// backward (Sec. 2.1 of the paper: the bandwidth-bound layers next to the convolutions; after a
// reconfiguration their cost scales with the compacted channel count).
//
// Both directions are two streaming passes: per-channel sums over all pixels (a column reduction: every
// thread keeps 8 consecutive channels = one 16-byte vector in registers for all the pixel rows it visits,
// workgroups own contiguous pixel ranges, partial sums go to a workspace and are combined in fp64 in a fixed
// order), then an element-wise pass with the per-channel constants in registers.  Sums are taken about a
// per-channel pivot (the first pixel) so that variance = E[d^2] - E[d]^2 does not cancel for channels whose
// mean is large against their spread.  No atomics: results are run-to-run identical.
//
// Algorithmic bytes per element: forward 2+2 read, 2 written; backward 4+4 read, 2 written.
#include "common.h"

namespace pt {

constexpr int kBnThreads = 256;
constexpr int kBnMaxC = 2048;      // 256 lanes x 8 channels
constexpr int kBnMaxBlocks = 1024;  // pixel ranges of the reduction passes

struct BnGeom {
    int64_t pixels;
    int C, cv, tx, ty;       // cv: 8-channel vectors per row; tx lanes across channels (>= cv), ty rows in flight
    int nblocks, rows_per_block;
};

inline BnGeom bn_geom(int64_t pixels, int C) {
    BnGeom g;
    g.pixels = pixels;
    g.C = C;
    g.cv = (C + 7) / 8;
    int tx = 1;
    while (tx < g.cv) tx <<= 1;
    g.tx = tx;
    g.ty = kBnThreads / tx;
    // at least 8 passes of ty rows per workgroup, at most kBnMaxBlocks workgroups
    int64_t rpb = (int64_t)g.ty * 8;
    if (ceil_div(pixels, rpb) > kBnMaxBlocks) rpb = round_up(ceil_div(pixels, kBnMaxBlocks), g.ty);
    g.rows_per_block = (int)rpb;
    g.nblocks = (int)ceil_div(pixels, rpb);
    return g;
}

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);
        f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

// MODE 0: a = sum (x - pivot), b = sum (x - pivot)^2.   MODE 1: a = sum dy, b = sum dy * xhat.
// partial layout: [2][nblocks][C].
template <int MODE>
__global__ __launch_bounds__(kBnThreads) void k_bn_sums(const uint16_t* __restrict__ x, int xpitch,
                                                        const uint16_t* __restrict__ dy, int dypitch, BnGeom g,
                                                        const float* __restrict__ mean, const float* __restrict__ invstd,
                                                        float* __restrict__ partial) {
    __shared__ float red[2][kBnThreads * 8];
    const int tid = threadIdx.x;
    const int tx = tid & (g.tx - 1), ty = tid / g.tx;
    const bool live = tx < g.cv;
    float c0[8], c1[8];  // MODE 0: pivot, unused.  MODE 1: mean, invstd
#pragma unroll
    for (int e = 0; e < 8; ++e) c0[e] = 0.f, c1[e] = 0.f;
    if (live) {
        if (MODE == 0) {
            unpack8(*reinterpret_cast<const uint4*>(x + tx * 8), c0);  // pixel 0 of every channel
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int c = tx * 8 + e;
                c0[e] = c < g.C ? mean[c] : 0.f;
                c1[e] = c < g.C ? invstd[c] : 0.f;
            }
        }
    }
    float a[8], b[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = 0.f, b[e] = 0.f;
    const int64_t r0 = (int64_t)blockIdx.x * g.rows_per_block;
    const int64_t r1 = min(g.pixels, r0 + g.rows_per_block);
    if (live) {
        for (int64_t r = r0 + ty; r < r1; r += g.ty) {
            float xv[8];
            unpack8(*reinterpret_cast<const uint4*>(x + r * xpitch + tx * 8), xv);
            if (MODE == 0) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float d = xv[e] - c0[e];
                    a[e] += d;
                    b[e] += d * d;
                }
            } else {
                float gv[8];
                unpack8(*reinterpret_cast<const uint4*>(dy + r * dypitch + tx * 8), gv);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    a[e] += gv[e];
                    b[e] += gv[e] * ((xv[e] - c0[e]) * c1[e]);
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        red[0][tid * 8 + e] = a[e];
        red[1][tid * 8 + e] = b[e];
    }
    __syncthreads();
    // row groups added in ty order: thread f owns channel f of the workgroup's tx*8 columns
    for (int f = tid; f < g.tx * 8; f += kBnThreads) {
        if (f >= g.C) continue;
        float s0 = 0.f, s1 = 0.f;
        for (int y = 0; y < g.ty; ++y) {
            s0 += red[0][(y * g.tx) * 8 + f];
            s1 += red[1][(y * g.tx) * 8 + f];
        }
        partial[(size_t)blockIdx.x * g.C + f] = s0;
        partial[((size_t)g.nblocks + blockIdx.x) * g.C + f] = s1;
    }
}

// 8 channels per workgroup, 32 threads per channel: each thread adds every 32nd workgroup partial in fp64 in
// ascending order (loads issued 8 at a time), the 32 slices are then added in slice order: a fixed order, so
// results are run-to-run identical.   MODE 0 -> mean, invstd.  MODE 1 -> dbeta (= a), dgamma (= b).
template <int MODE>
__global__ __launch_bounds__(256) void k_bn_finish(const float* __restrict__ partial, const uint16_t* __restrict__ x,
                                                   BnGeom g, float eps, float* __restrict__ out0,
                                                   float* __restrict__ out1) {
    __shared__ double red[2][32][8];
    const int cx = threadIdx.x & 7, sl = threadIdx.x >> 3;
    const int c = blockIdx.x * 8 + cx;
    double s0 = 0.0, s1 = 0.0;
    if (c < g.C) {
        const float* pa = partial + c;
        const float* pb = partial + (size_t)g.nblocks * g.C + c;
        for (int b = sl; b < g.nblocks; b += 32 * 8) {
            float va[8], vb[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                // unconditional loads from a clamped row (so that all 16 are in flight together), masked after
                const int bb = b + 32 * u;
                const size_t row = (size_t)min(bb, g.nblocks - 1) * g.C;
                va[u] = pa[row];
                vb[u] = pb[row];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (b + 32 * u >= g.nblocks) va[u] = 0.f, vb[u] = 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                s0 += (double)va[u];
                s1 += (double)vb[u];
            }
        }
    }
    red[0][sl][cx] = s0;
    red[1][sl][cx] = s1;
    __syncthreads();
    if (sl != 0 || c >= g.C) return;
    s0 = 0.0, s1 = 0.0;
    for (int i = 0; i < 32; ++i) {
        s0 += red[0][i][cx];
        s1 += red[1][i][cx];
    }
    if (MODE == 0) {
        const double pivot = x ? (double)__uint_as_float((uint32_t)x[c] << 16) : 0.0;  // no x: plain sums
        const double m = s0 / (double)g.pixels;           // mean of (x - pivot)
        double var = s1 / (double)g.pixels - m * m;       // biased variance
        if (var < 0.0) var = 0.0;
        out0[c] = (float)(pivot + m);
        out1[c] = (float)(1.0 / sqrt(var + (double)eps));
    } else {
        out0[c] = (float)s0;
        out1[c] = (float)s1;
    }
}

// MODE 0: y = (x - mean) * (gamma * invstd) + beta.
// MODE 1: dx = (gamma * invstd) * (dy - dbeta/M - xhat * dgamma/M).
template <int MODE>
__global__ __launch_bounds__(kBnThreads) void k_bn_apply(const uint16_t* __restrict__ x, int xpitch,
                                                         const uint16_t* __restrict__ dy, int dypitch, BnGeom g,
                                                         const float* __restrict__ mean, const float* __restrict__ invstd,
                                                         const float* __restrict__ p0, const float* __restrict__ p1,
                                                         const float* __restrict__ gamma, uint16_t* __restrict__ out,
                                                         int opitch) {
    const int tid = threadIdx.x;
    const int tx = tid & (g.tx - 1), ty = tid / g.tx;
    if (tx >= g.cv) return;
    float mu[8], sc[8], k0[8], k1[8];  // MODE 0: k0 = beta.  MODE 1: k0 = dbeta/M, k1 = invstd * dgamma/M
    const float invM = 1.0f / (float)g.pixels;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int c = min(tx * 8 + e, g.C - 1);
        mu[e] = mean[c];
        sc[e] = gamma[c] * invstd[c];
        if (MODE == 0) {
            k0[e] = p0[c];
            k1[e] = 0.f;
        } else {
            k0[e] = p0[c] * invM;
            k1[e] = invstd[c] * (p1[c] * invM);
        }
    }
    // Padding channels of the last vector go out as zero: whole rows are written, never partial ones (a hole in
    // every row costs the memory system a merge of partial lines and halves the store rate).
    const int nlast = g.C - tx * 8;  // valid channels of this thread's vector (>= 8: all)
    auto halves = [&](int k) { return (k < nlast ? 0xFFFFu : 0u) | (k + 1 < nlast ? 0xFFFF0000u : 0u); };
    const uint32_t m0 = halves(0), m1 = halves(2), m2 = halves(4), m3 = halves(6);
    const int64_t stride = (int64_t)gridDim.x * g.ty;
    // last pixels first: the reduction pass before this one ended there, so they are the likeliest to still sit
    // in the chip's caches
    for (int64_t q = (int64_t)blockIdx.x * g.ty + ty; q < g.pixels; q += stride) {
        const int64_t r = g.pixels - 1 - q;
        float xv[8], o[8];
        unpack8(*reinterpret_cast<const uint4*>(x + r * xpitch + tx * 8), xv);
        if (MODE == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (xv[e] - mu[e]) * sc[e] + k0[e];
        } else {
            float gv[8];
            unpack8(*reinterpret_cast<const uint4*>(dy + r * dypitch + tx * 8), gv);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = sc[e] * (gv[e] - k0[e] - (xv[e] - mu[e]) * k1[e]);
        }
        uint4 pk;
        pk.x = cvt_pk_bf16(o[0], o[1]) & m0;
        pk.y = cvt_pk_bf16(o[2], o[3]) & m1;
        pk.z = cvt_pk_bf16(o[4], o[5]) & m2;
        pk.w = cvt_pk_bf16(o[6], o[7]) & m3;
        *reinterpret_cast<uint4*>(out + r * opitch + tx * 8) = pk;
    }
}

}  // namespace pt

using namespace pt;

static int32_t bn_check(int64_t pixels, int32_t C, int32_t p0, int32_t p1, int32_t p2) {
    if (pixels <= 0 || C <= 0 || p0 < C || p1 < C || p2 < C) return PT_ERR_SHAPE;
    if (C > kBnMaxC || pixels > 0x7fffffff) return PT_ERR_UNSUPPORTED;
    if (p0 % 8 || p1 % 8 || p2 % 8) return PT_ERR_UNSUPPORTED;  // 16-byte rows only
    return PT_OK;
}
static bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

extern "C" int32_t pt_bn_workspace_bytes(int64_t pixels, int32_t C, size_t* bytes) {
    if (!bytes) return PT_ERR_NULL;
    const int32_t rc = bn_check(pixels, C, (C + 7) & ~7, (C + 7) & ~7, (C + 7) & ~7);
    if (rc != PT_OK) return rc;
    const BnGeom g = bn_geom(pixels, C);
    *bytes = (size_t)round_up((int64_t)2 * g.nblocks * C * 4, 256);
    return PT_OK;
}

extern "C" int32_t pt_bn_fwd(const uint16_t* x, int64_t pixels, int32_t C, int32_t x_cpitch, const float* gamma,
                             const float* beta, float eps, uint16_t* y, int32_t y_cpitch, float* mean, float* invstd,
                             void* ws, size_t ws_bytes, void* stream) {
    int32_t rc = bn_check(pixels, C, x_cpitch, y_cpitch, x_cpitch);
    if (rc != PT_OK) return rc;
    if (!(eps >= 0.f)) return PT_ERR_SHAPE;
    if (!x || !gamma || !beta || !y || !mean || !invstd || !ws) return PT_ERR_NULL;
    if (!al16(x) || !al16(y) || !al16(ws)) return PT_ERR_UNSUPPORTED;
    const BnGeom g = bn_geom(pixels, C);
    if (ws_bytes < (size_t)2 * g.nblocks * C * 4) return PT_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    float* part = (float*)ws;
    hipLaunchKernelGGL(k_bn_sums<0>, dim3(g.nblocks), dim3(kBnThreads), 0, st, x, x_cpitch, (const uint16_t*)nullptr, 0, g,
                       (const float*)nullptr, (const float*)nullptr, part);
    rc = launch_status();
    if (rc != PT_OK) return rc;
    hipLaunchKernelGGL(k_bn_finish<0>, dim3((unsigned)ceil_div(C, 8)), dim3(256), 0, st, part, x, g, eps, mean, invstd);
    rc = launch_status();
    if (rc != PT_OK) return rc;
    const int64_t passes = ceil_div(pixels, g.ty);
    const unsigned grid = (unsigned)(passes < 256 * 8 ? passes : 256 * 8);
    hipLaunchKernelGGL(k_bn_apply<0>, dim3(grid), dim3(kBnThreads), 0, st, x, x_cpitch, (const uint16_t*)nullptr, 0, g, mean,
                       invstd, beta, (const float*)nullptr, gamma, y, y_cpitch);
    return launch_status();
}

extern "C" int32_t pt_bn_bwd(const uint16_t* x, const uint16_t* dy, int64_t pixels, int32_t C, int32_t x_cpitch,
                             int32_t dy_cpitch, const float* gamma, const float* mean, const float* invstd, uint16_t* dx,
                             int32_t dx_cpitch, float* dgamma, float* dbeta, void* ws, size_t ws_bytes, void* stream) {
    int32_t rc = bn_check(pixels, C, x_cpitch, dy_cpitch, dx_cpitch);
    if (rc != PT_OK) return rc;
    if (!x || !dy || !gamma || !mean || !invstd || !dx || !dgamma || !dbeta || !ws) return PT_ERR_NULL;
    if (!al16(x) || !al16(dy) || !al16(dx) || !al16(ws)) return PT_ERR_UNSUPPORTED;
    const BnGeom g = bn_geom(pixels, C);
    if (ws_bytes < (size_t)2 * g.nblocks * C * 4) return PT_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    float* part = (float*)ws;
    hipLaunchKernelGGL(k_bn_sums<1>, dim3(g.nblocks), dim3(kBnThreads), 0, st, x, x_cpitch, dy, dy_cpitch, g, mean, invstd,
                       part);
    rc = launch_status();
    if (rc != PT_OK) return rc;
    hipLaunchKernelGGL(k_bn_finish<1>, dim3((unsigned)ceil_div(C, 8)), dim3(256), 0, st, part, x, g, 0.f, dbeta, dgamma);
    rc = launch_status();
    if (rc != PT_OK) return rc;
    const int64_t passes = ceil_div(pixels, g.ty);
    const unsigned grid = (unsigned)(passes < 256 * 8 ? passes : 256 * 8);
    hipLaunchKernelGGL(k_bn_apply<1>, dim3(grid), dim3(kBnThreads), 0, st, x, x_cpitch, dy, dy_cpitch, g, mean, invstd, dbeta,
                       dgamma, gamma, dx, dx_cpitch);
    return launch_status();
}

// Normalisation whose statistics pass was done by the producing convolution (pt_conv_fwd_stats): finish + apply.
extern "C" int32_t pt_bn_fwd_from_sums(const uint16_t* x, int64_t pixels, int32_t C, int32_t x_cpitch, const float* sums,
                                       int32_t n_partial, const float* gamma, const float* beta, float eps, uint16_t* y,
                                       int32_t y_cpitch, float* mean, float* invstd, void* stream) {
    int32_t rc = bn_check(pixels, C, x_cpitch, y_cpitch, x_cpitch);
    if (rc != PT_OK) return rc;
    if (!(eps >= 0.f) || n_partial <= 0) return PT_ERR_SHAPE;
    if (!x || !sums || !gamma || !beta || !y || !mean || !invstd) return PT_ERR_NULL;
    if (!al16(x) || !al16(y)) return PT_ERR_UNSUPPORTED;
    BnGeom g = bn_geom(pixels, C);
    g.nblocks = n_partial;  // rows of `sums` per statistic
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(k_bn_finish<0>, dim3((unsigned)ceil_div(C, 8)), dim3(256), 0, st, sums, (const uint16_t*)nullptr, g,
                       eps, mean, invstd);
    rc = launch_status();
    if (rc != PT_OK) return rc;
    const int64_t passes = ceil_div(pixels, g.ty);
    const unsigned grid = (unsigned)(passes < 256 * 8 ? passes : 256 * 8);
    hipLaunchKernelGGL(k_bn_apply<0>, dim3(grid), dim3(kBnThreads), 0, st, x, x_cpitch, (const uint16_t*)nullptr, 0, g, mean,
                       invstd, beta, (const float*)nullptr, gamma, y, y_cpitch);
    return launch_status();
}
