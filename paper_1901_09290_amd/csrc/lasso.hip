// Channel group-lasso kernels (Eq. 1-2): group L2 norms (+ bf16 shadow weights) and the gradient.
//
// Both are HBM-bound: group_norms reads the fp32 master weights once (4 B/param, +2 B/param written
// when the bf16 shadow is emitted); the gradient pass reads w and dw and writes dw (12 B/param).
//
// Thread layout (both kernels): a workgroup of 256 threads is a TY x TX grid, TX = lanes across the
// channel axis (a power of two <= 64, so a row of TX lanes lives inside one wavefront), TY = 256/TX
// rows in flight.  A thread keeps the same channel columns for every row it visits, so input-channel
// (column) sums stay in registers; output-channel (row) sums are reduced across the TX lanes with
// wavefront shuffles and then across rows through LDS.  All reductions run in a fixed order.
#include "common.h"

namespace pt {

constexpr int kNormThreads = 256;
constexpr int kNormMaxRows = 2048;  // LDS row-sum slots per workgroup
constexpr int kNormColsPerThread = 8;

template <int VEC>
struct VecT;
template <>
struct VecT<4> {
    using type = float4;
};
template <>
struct VecT<1> {
    using type = float;
};

template <int VEC>
__device__ __forceinline__ void load_vec(const float* p, float (&v)[VEC]) {
    if constexpr (VEC == 4) {
        float4 t = *reinterpret_cast<const float4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = *p;
    }
}

// One workgroup = filters [k0, k0 + fpb).  Writes out_norm for its filters and one row of column
// partial sums (sum of squares per input channel over its filters) to ws_cols[block][C].
template <int VEC>
__global__ __launch_bounds__(kNormThreads) void k_group_norms_partial(const float* __restrict__ w, int K, int RS,
                                                                      int C, int cpitch, int fpb, int txlog2,
                                                                      uint16_t* __restrict__ shadow,
                                                                      float* __restrict__ out_norm,
                                                                      float* __restrict__ ws_cols) {
    __shared__ float rowsum[kNormMaxRows];
    __shared__ float colred[kNormThreads * kNormColsPerThread * VEC];
    const int tid = threadIdx.x;
    const int TX = 1 << txlog2, TY = kNormThreads >> txlog2;
    const int tx = tid & (TX - 1), ty = tid >> txlog2;
    const int k0 = blockIdx.x * fpb;
    const int k1 = min(K, k0 + fpb);
    const int nrows = (k1 - k0) * RS;
    const size_t rowbase = (size_t)k0 * RS;
    const int Lv = (C + VEC - 1) / VEC;

    for (int r = tid; r < nrows; r += kNormThreads) rowsum[r] = 0.f;
    __syncthreads();

    for (int cbase = 0; cbase < Lv; cbase += TX * kNormColsPerThread) {
        float acc[kNormColsPerThread][VEC];
#pragma unroll
        for (int j = 0; j < kNormColsPerThread; ++j)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[j][e] = 0.f;

        for (int r = ty; r < nrows; r += TY) {
            const size_t roff = (rowbase + r) * (size_t)cpitch;
            float rs = 0.f;
#pragma unroll
            for (int j = 0; j < kNormColsPerThread; ++j) {
                const int cg = cbase + tx + j * TX;
                if (cg < Lv) {
                    float v[VEC];
                    load_vec<VEC>(w + roff + (size_t)cg * VEC, v);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        if (cg * VEC + e >= C) v[e] = 0.f;  // pitch padding is not data
                        const float q = v[e] * v[e];
                        acc[j][e] += q;
                        rs += q;
                    }
                    if (shadow) {
                        if constexpr (VEC == 4) {
                            if (cg * 4 + 3 < C) {
                                uint2 o;
                                o.x = pack_bf16x2(v[0], v[1]);
                                o.y = pack_bf16x2(v[2], v[3]);
                                *reinterpret_cast<uint2*>(shadow + roff + (size_t)cg * 4) = o;
                            } else {
                                for (int e = 0; e < 4; ++e)
                                    if (cg * 4 + e < C) shadow[roff + (size_t)cg * 4 + e] = f32_to_bf16(v[e]);
                            }
                        } else {
                            shadow[roff + cg] = f32_to_bf16(v[0]);
                        }
                    }
                }
            }
            for (int off = TX >> 1; off > 0; off >>= 1) rs += __shfl_xor(rs, off);
            if (tx == 0) rowsum[r] += rs;  // always the same thread for a given row: fixed order
        }

        // column sums: across the TY row groups, in ty order
#pragma unroll
        for (int j = 0; j < kNormColsPerThread; ++j)
#pragma unroll
            for (int e = 0; e < VEC; ++e) colred[((ty * kNormColsPerThread + j) * TX + tx) * VEC + e] = acc[j][e];
        __syncthreads();
        const int slots = kNormColsPerThread * TX * VEC;
        for (int f = tid; f < slots; f += kNormThreads) {
            const int c = cbase * VEC + f;  // (j*TX + tx)*VEC + e is the column offset inside this chunk
            if (c < C) {
                float s = 0.f;
                for (int y = 0; y < TY; ++y) s += colred[y * slots + f];
                ws_cols[(size_t)blockIdx.x * C + c] = s;
            }
        }
        __syncthreads();
    }

    for (int kk = tid; kk < k1 - k0; kk += kNormThreads) {
        float s = 0.f;
        for (int j = 0; j < RS; ++j) s += rowsum[kk * RS + j];
        out_norm[k0 + kk] = sqrtf(s);
    }
}

__global__ void k_group_norms_finish(const float* __restrict__ ws_cols, int nblk, int C, float* __restrict__ in_norm) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    float s = 0.f;
    for (int b = 0; b < nblk; ++b) s += ws_cols[(size_t)b * C + c];
    in_norm[c] = sqrtf(s);
}

template <int VEC>
__global__ __launch_bounds__(kNormThreads) void k_group_lasso_grad(const float* __restrict__ w,
                                                                   const float* __restrict__ out_norm,
                                                                   const float* __restrict__ in_norm, float lambda,
                                                                   uint32_t flags, float* __restrict__ dw,
                                                                   int64_t rows, int RS, int C, int cpitch,
                                                                   int rows_per_block, int txlog2) {
    const int tid = threadIdx.x;
    const int TX = 1 << txlog2, TY = kNormThreads >> txlog2;
    const int tx = tid & (TX - 1), ty = tid >> txlog2;
    const int Lv = (C + VEC - 1) / VEC;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = min(rows, r0 + rows_per_block);
    const bool reg_out = flags & PT_LASSO_OUT, reg_in = flags & PT_LASSO_IN;

    for (int cg = tx; cg < Lv; cg += TX) {
        float inv_in[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const int c = cg * VEC + e;
            const float nrm = (reg_in && c < C) ? in_norm[c] : 0.f;
            inv_in[e] = nrm > 0.f ? 1.0f / nrm : 0.f;
        }
        for (int64_t r = r0 + ty; r < r1; r += TY) {
            const int k = (int)(r / RS);
            const float on = reg_out ? out_norm[k] : 0.f;
            const float inv_out = on > 0.f ? 1.0f / on : 0.f;
            const size_t off = (size_t)r * cpitch + (size_t)cg * VEC;
            float v[VEC], g[VEC];
            load_vec<VEC>(w + off, v);
            load_vec<VEC>(dw + off, g);
#pragma unroll
            for (int e = 0; e < VEC; ++e) g[e] += lambda * (v[e] * (inv_out + inv_in[e]));
            if constexpr (VEC == 4) {
                if (cg * 4 + 3 < C) {
                    *reinterpret_cast<float4*>(dw + off) = make_float4(g[0], g[1], g[2], g[3]);
                } else {
                    for (int e = 0; e < 4; ++e)
                        if (cg * 4 + e < C) dw[off + e] = g[e];
                }
            } else {
                dw[off] = g[0];
            }
        }
    }
}

static int tx_log2_for(int Lv) {
    int l = 0;
    while ((1 << l) < Lv && l < 6) ++l;
    return l;
}

static int norms_fpb(int K, int RS, int C) {
    int64_t per_filter = (int64_t)RS * C;
    int64_t fpb = 32768 / (per_filter > 0 ? per_filter : 1);
    if (fpb < 1) fpb = 1;
    if (fpb > kNormMaxRows / RS) fpb = kNormMaxRows / RS;
    if (fpb < 1) fpb = 1;
    if (fpb > K) fpb = K;
    return (int)fpb;
}

}  // namespace pt

using namespace pt;

extern "C" int32_t pt_group_norms_workspace_bytes(int32_t K, int32_t RS, int32_t C, size_t* bytes) {
    if (!bytes) return PT_ERR_NULL;
    if (K <= 0 || RS <= 0 || C <= 0) return PT_ERR_SHAPE;
    if (RS > kNormMaxRows || C > 16384) return PT_ERR_UNSUPPORTED;
    const int fpb = norms_fpb(K, RS, C);
    const int64_t nblk = ceil_div(K, fpb);
    *bytes = (size_t)round_up(nblk * (int64_t)C * 4, 256);
    return PT_OK;
}

extern "C" int32_t pt_group_norms(const float* w, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch, float* out_norm,
                                  float* in_norm, uint16_t* w_shadow, void* ws, size_t ws_bytes, void* stream) {
    if (!w || !out_norm || !in_norm || !ws) return PT_ERR_NULL;
    if (K <= 0 || RS <= 0 || C <= 0 || w_cpitch < C) return PT_ERR_SHAPE;
    size_t need = 0;
    int32_t rc = pt_group_norms_workspace_bytes(K, RS, C, &need);
    if (rc != PT_OK) return rc;
    if (ws_bytes < need) return PT_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int fpb = norms_fpb(K, RS, C);
    const int nblk = (int)ceil_div(K, fpb);
    const bool vec = (w_cpitch % 4 == 0) && (((uintptr_t)w & 15) == 0) &&
                     (!w_shadow || ((uintptr_t)w_shadow & 7) == 0);
    float* cols = (float*)ws;
    if (vec) {
        const int txl = tx_log2_for((C + 3) / 4);
        hipLaunchKernelGGL(k_group_norms_partial<4>, dim3(nblk), dim3(kNormThreads), 0, st, w, K, RS, C, w_cpitch, fpb,
                           txl, w_shadow, out_norm, cols);
    } else {
        const int txl = tx_log2_for(C);
        hipLaunchKernelGGL(k_group_norms_partial<1>, dim3(nblk), dim3(kNormThreads), 0, st, w, K, RS, C, w_cpitch, fpb,
                           txl, w_shadow, out_norm, cols);
    }
    rc = launch_status();
    if (rc != PT_OK) return rc;
    hipLaunchKernelGGL(k_group_norms_finish, dim3((C + 255) / 256), dim3(256), 0, st, cols, nblk, C, in_norm);
    return launch_status();
}

extern "C" int32_t pt_group_lasso_grad(const float* w, const float* out_norm, const float* in_norm, float lambda,
                                       uint32_t flags, float* dw, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch,
                                       void* stream) {
    if (!w || !out_norm || !in_norm || !dw) return PT_ERR_NULL;
    if (K <= 0 || RS <= 0 || C <= 0 || w_cpitch < C) return PT_ERR_SHAPE;
    if (flags & ~3u) return PT_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    const int64_t rows = (int64_t)K * RS;
    const bool vec = (w_cpitch % 4 == 0) && (((uintptr_t)w & 15) == 0) && (((uintptr_t)dw & 15) == 0);
    const int Lv = vec ? (C + 3) / 4 : C;
    const int txl = tx_log2_for(Lv);
    // about 8192 vectors per workgroup
    int64_t rpb = ceil_div(8192, Lv);
    const int TY = kNormThreads >> txl;
    rpb = round_up(rpb, TY);
    const int64_t nblk = ceil_div(rows, rpb);
    if (nblk > 0x7fffffff) return PT_ERR_UNSUPPORTED;
    if (vec)
        hipLaunchKernelGGL(k_group_lasso_grad<4>, dim3((unsigned)nblk), dim3(kNormThreads), 0, st, w, out_norm, in_norm,
                           lambda, flags, dw, rows, RS, C, w_cpitch, (int)rpb, txl);
    else
        hipLaunchKernelGGL(k_group_lasso_grad<1>, dim3((unsigned)nblk), dim3(kNormThreads), 0, st, w, out_norm, in_norm,
                           lambda, flags, dw, rows, RS, C, w_cpitch, (int)rpb, txl);
    return launch_status();
}
