// Channel group-lasso kernels (Eq. 1-2): group L2 norms (+ bf16 shadow weights) and the gradient.
//
// Both are HBM-bound: group_norms reads the fp32 master weights once (4 B/param, +2 B/param written
// when the bf16 shadow is emitted); the gradient pass reads w and dw and writes dw (12 B/param).
// A network has tens of layers whose weight tensors are small (KBs to a few MB), so every kernel here
// is multi-tensor: up to kMaxJobs layers ride in the kernel arguments of ONE launch and a workgroup
// finds its (layer, row chunk) from a table of first-workgroup indices.
//
// Thread layout: a workgroup of 256 threads is a TY x TX grid, TX = lanes across the channel axis (a
// power of two <= 64, so a row of TX lanes lives inside one wavefront), TY = 256/TX rows in flight.  A
// thread keeps the same channel columns for every row it visits, so input-channel (column) sums stay
// in registers; output-channel (row) sums are reduced across the TX lanes with wavefront shuffles.
// Two levels, fixed order, no atomics: a workgroup owns whole rows of a chunk and writes one
// sum-of-squares per row and one partial per column; the finish kernel adds the R*S row sums of each
// filter and the per-chunk column partials in ascending order.
#include <vector>
#include "common.h"
#include "norms.h"

namespace pt {

constexpr int kThreads = 256;
constexpr int kMaxC = 2048;  // 64 lanes x (8 float4 column groups | 32 scalar column groups) per thread
#ifndef PT_NORM_JOBS
#define PT_NORM_JOBS 64  // 64 x 88 bytes + 16 = 5.5 KiB of kernel arguments
#endif
constexpr int kMaxJobs = PT_NORM_JOBS;  // layers per launch (the table rides in the kernel arguments)

struct NormJob {
    const float* w;
    uint16_t* shadow;   // nullptr: no bf16 copy
    float* out_norm;
    float* in_norm;
    uint8_t* zero_out;  // nullptr, or [K]: the finish pass also writes (out_norm < thr)
    uint8_t* zero_in;   // nullptr, or [C]
    uint32_t ws_off;    // this job's scratch in the workspace, in floats: [K*RS] row sums, then [n_chunks][C] column partials
    int K, RS, C, cpitch;
    int first_block, n_chunks, rows_per_chunk;
    int fin_first;      // first workgroup of this job in the finish kernel
};
struct NormJobs {
    NormJob j[kMaxJobs];
    float* ws;
    float thr;
    int n;
};
static_assert(sizeof(NormJobs) <= 8192, "kernel-argument table");

struct LassoJob {
    const float* w;
    const float* out_norm;
    const float* in_norm;
    float* dw;
    float* mom;  // optimizer step only: momentum buffer; then w is updated in place and dw is read-only
    int K, RS, C, cpitch;
    int first_block, n_chunks, rows_per_chunk, txlog2;
    uint32_t flags;
    int pad;
};
constexpr int kMaxLassoJobs = 32;
struct LassoJobs {
    LassoJob j[kMaxLassoJobs];
    int n;
};

// Last job whose first workgroup is <= block (the table is ascending); uniform, so it runs on the scalar unit.
template <typename Jobs>
__device__ __forceinline__ int find_job(const Jobs& jobs, int block) {
    int lo = 0, hi = jobs.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs.j[mid].first_block <= block) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

template <int VEC>
__device__ __forceinline__ void load_vec(const float* p, float (&v)[VEC]) {
    if constexpr (VEC == 4) {
        float4 t = *reinterpret_cast<const float4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = *p;
    }
}

// Channel-axis layout of a layer for the vector kernel: Lv float4 columns, CG = 1 << cglog2 column groups per
// thread (1, 2, 4 or 8), TX = 1 << txlog2 lanes across a row; column of (tx, j) = tx + j * TX.
struct NormLayout {
    int cglog2, txlog2;
};
__host__ __device__ inline NormLayout norm_layout(int C) {
    const int Lv = (C + 3) >> 2;
    NormLayout l;
    l.cglog2 = 0;
    while ((64 << l.cglog2) < Lv) ++l.cglog2;           // <= 3 for C <= 2048
    const int per = (Lv + (1 << l.cglog2) - 1) >> l.cglog2;  // columns per group
    l.txlog2 = 0;
    while ((1 << l.txlog2) < per) ++l.txlog2;            // <= 6
    return l;
}

// One workgroup = one chunk of whole rows of one layer (vector path: 16-byte aligned rows).  A thread keeps eight
// 16-byte loads in flight: 8 / CG rows at a time, CG column groups each.  Row sums: per thread over its columns,
// then a shuffle tree over the TX lanes of the row.  Column sums: in registers over the rows a thread visits, then
// over the rows of a wavefront by shuffles and over the four wavefronts through LDS, all in a fixed order.
template <int CG>
__device__ __forceinline__ void norms_partial_body(const NormJob& J, float* __restrict__ ws, int chunk, int txlog2,
                                                   float (*colred)[1024]) {
    constexpr int U = 8 / CG;  // rows in flight per thread
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int TX = 1 << txlog2, TY = kThreads >> txlog2;
    const int tx = tid & (TX - 1), ty = tid >> txlog2;
    const int64_t rows = (int64_t)J.K * J.RS;
    const int64_t r0 = (int64_t)chunk * J.rows_per_chunk;
    const int64_t r1 = min(rows, r0 + J.rows_per_chunk);
    const int C = J.C, cpitch = J.cpitch;
    const int Lv = (C + 3) >> 2;
    const float* __restrict__ w = J.w;
    uint16_t* __restrict__ shadow = J.shadow;
    float* __restrict__ rowsq = ws + J.ws_off;
    float* __restrict__ colpart = rowsq + rows;

    float acc[CG][4];
    bool col_ok[CG];
    int col_n[CG];  // valid elements of this thread's j-th column vector (0: none)
#pragma unroll
    for (int j = 0; j < CG; ++j) {
        const int cg = tx + j * TX;
        col_ok[j] = cg < Lv;
        col_n[j] = col_ok[j] ? min(4, C - cg * 4) : 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[j][e] = 0.f;
    }

    for (int64_t rb = r0 + ty; rb < r1; rb += (int64_t)TY * U) {
        float4 v[U][CG];
        // all loads first (rows past the chunk and columns past the row re-read a valid vector and are masked below)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t r = min(rb + (int64_t)u * TY, r1 - 1);
#pragma unroll
            for (int j = 0; j < CG; ++j) {
                const int cg = col_ok[j] ? tx + j * TX : 0;
                v[u][j] = *reinterpret_cast<const float4*>(w + (size_t)r * cpitch + (size_t)cg * 4);
            }
        }
        float rs[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t r = rb + (int64_t)u * TY;
            const bool row_ok = r < r1;
            rs[u] = 0.f;
#pragma unroll
            for (int j = 0; j < CG; ++j) {
                float e4[4] = {v[u][j].x, v[u][j].y, v[u][j].z, v[u][j].w};
                const int n = row_ok ? col_n[j] : 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x = e < n ? e4[e] : 0.f;  // pitch padding is not data
                    e4[e] = x;
                    const float q = x * x;
                    acc[j][e] += q;
                    rs[u] += q;
                }
                if (shadow && n > 0) {
                    const size_t off = (size_t)r * cpitch + (size_t)(tx + j * TX) * 4;
                    if (n == 4) {
                        uint2 o;
                        o.x = cvt_pk_bf16(e4[0], e4[1]);
                        o.y = cvt_pk_bf16(e4[2], e4[3]);
                        *reinterpret_cast<uint2*>(shadow + off) = o;
                    } else {
                        for (int e = 0; e < n; ++e) shadow[off + e] = f32_to_bf16(e4[e]);
                    }
                }
            }
        }
        for (int off = TX >> 1; off > 0; off >>= 1) {
#pragma unroll
            for (int u = 0; u < U; ++u) rs[u] += __shfl_xor(rs[u], off);
        }
        if (tx == 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t r = rb + (int64_t)u * TY;
                if (r < r1) rowsq[r] = rs[u];
            }
        }
    }

    // column partials: rows of one wavefront by shuffles (lanes tx, tx + TX, ... hold the same columns) ...
    for (int off = TX; off < 64; off <<= 1) {
#pragma unroll
        for (int j = 0; j < CG; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[j][e] += __shfl_xor(acc[j][e], off);
    }
    // ... then the four wavefronts through LDS in wavefront order, at most four column groups (1024 floats) per round
    constexpr int ROUNDS = CG > 4 ? CG / 4 : 1, PER = CG > 4 ? 4 : CG;
#pragma unroll
    for (int rnd = 0; rnd < ROUNDS; ++rnd) {
        if (rnd > 0) __syncthreads();
        if (lane < TX) {
#pragma unroll
            for (int jj = 0; jj < PER; ++jj)
#pragma unroll
                for (int e = 0; e < 4; ++e) colred[wave][(jj * TX + lane) * 4 + e] = acc[rnd * PER + jj][e];
        }
        __syncthreads();
        // with fewer than 64 lanes per row every wavefront holds full sums of its own rows; all four are added
        for (int f = tid; f < PER * TX * 4; f += kThreads) {
            const int c = rnd * PER * TX * 4 + f;
            if (c < C) colpart[(size_t)chunk * C + c] = ((colred[0][f] + colred[1][f]) + colred[2][f]) + colred[3][f];
        }
    }
}

__global__ __launch_bounds__(kThreads) void k_group_norms_partial_vec(const NormJobs jobs) {
    __shared__ float colred[4][1024];
    const int ji = find_job(jobs, blockIdx.x);
    const NormJob& J = jobs.j[ji];
    const int chunk = blockIdx.x - J.first_block;
    const NormLayout l = norm_layout(J.C);
    switch (l.cglog2) {  // uniform
        case 0: norms_partial_body<1>(J, jobs.ws, chunk, l.txlog2, colred); break;
        case 1: norms_partial_body<2>(J, jobs.ws, chunk, l.txlog2, colred); break;
        case 2: norms_partial_body<4>(J, jobs.ws, chunk, l.txlog2, colred); break;
        default: norms_partial_body<8>(J, jobs.ws, chunk, l.txlog2, colred); break;
    }
}

// Element-wise path (rows that are not 16-byte aligned): one element per lane and column group, one row at a time.
__global__ __launch_bounds__(kThreads) void k_group_norms_partial_elem(const NormJobs jobs) {
    constexpr int kColsPerThread = kMaxC / 64;
    __shared__ float colred[kThreads];
    const int ji = find_job(jobs, blockIdx.x);
    const NormJob& J = jobs.j[ji];
    const int chunk = blockIdx.x - J.first_block;
    const int tid = threadIdx.x;
    int txlog2 = 0;
    while ((1 << txlog2) < J.C && txlog2 < 6) ++txlog2;
    const int TX = 1 << txlog2, TY = kThreads >> txlog2;
    const int tx = tid & (TX - 1), ty = tid >> txlog2;
    const int64_t rows = (int64_t)J.K * J.RS;
    const int64_t r0 = (int64_t)chunk * J.rows_per_chunk;
    const int64_t r1 = min(rows, r0 + J.rows_per_chunk);
    const int C = J.C, cpitch = J.cpitch;
    const float* __restrict__ w = J.w;
    uint16_t* __restrict__ shadow = J.shadow;
    float* __restrict__ rowsq = jobs.ws + J.ws_off;
    float* __restrict__ colpart = rowsq + rows;

    float acc[kColsPerThread];
#pragma unroll
    for (int j = 0; j < kColsPerThread; ++j) acc[j] = 0.f;
    for (int64_t r = r0 + ty; r < r1; r += TY) {
        const size_t roff = (size_t)r * cpitch;
        float rs = 0.f;
#pragma unroll
        for (int j = 0; j < kColsPerThread; ++j) {
            const int c = tx + j * TX;
            if (c < C) {
                const float v = w[roff + c];
                const float q = v * v;
                acc[j] += q;
                rs += q;
                if (shadow) shadow[roff + c] = f32_to_bf16(v);
            }
        }
        for (int off = TX >> 1; off > 0; off >>= 1) rs += __shfl_xor(rs, off);
        if (tx == 0) rowsq[r] = rs;
    }
    // column partials: across the TY row groups of the workgroup, in ty order, one column group at a time
#pragma unroll
    for (int j = 0; j < kColsPerThread; ++j) {
        if (j * TX >= C) break;  // uniform
        __syncthreads();
        colred[ty * TX + tx] = acc[j];
        __syncthreads();
        for (int f = tid; f < TX; f += kThreads) {
            const int c = j * TX + f;
            if (c < C) {
                float s = 0.f;
                for (int y = 0; y < TY; ++y) s += colred[y * TX + f];
                colpart[(size_t)chunk * C + c] = s;
            }
        }
    }
}

// Sixteen lanes per group (K filters, then C input channels of each job): the lanes stride over the R*S row
// sums of a filter / the per-chunk partials of a channel, then a fixed shuffle tree adds the 16 lane sums.
// The order of additions depends only on the shapes, so results are run-to-run identical.  Jobs with mask
// pointers also get their zero masks here: zero[g] = (norm[g] < thr), the comparison of pt_zero_groups.
constexpr int kFinLanes = 16, kFinGroups = kThreads / kFinLanes;
__global__ __launch_bounds__(kThreads) void k_group_norms_finish(const NormJobs jobs) {
    int lo = 0, hi = jobs.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs.j[mid].fin_first <= (int)blockIdx.x) lo = mid;
        else hi = mid - 1;
    }
    const NormJob& J = jobs.j[lo];
    const float* __restrict__ rowsq = jobs.ws + J.ws_off;
    const float* __restrict__ colpart = rowsq + (int64_t)J.K * J.RS;
    const int l = threadIdx.x & (kFinLanes - 1);
    const int g = (blockIdx.x - J.fin_first) * kFinGroups + (threadIdx.x / kFinLanes);
    const bool live = g < J.K + J.C;
    float s = 0.f;
    if (live && g < J.K) {
        for (int t = l; t < J.RS; t += kFinLanes) s += rowsq[(size_t)g * J.RS + t];
    } else if (live) {
        const int c = g - J.K;
        for (int b = l; b < J.n_chunks; b += kFinLanes) s += colpart[(size_t)b * J.C + c];
    }
    for (int off = kFinLanes / 2; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (live && l == 0) {
        const float nrm = sqrtf(s);
        if (g < J.K) {
            J.out_norm[g] = nrm;
            if (J.zero_out) J.zero_out[g] = nrm < jobs.thr ? 1 : 0;
        } else {
            J.in_norm[g - J.K] = nrm;
            if (J.zero_in) J.zero_in[g - J.K] = nrm < jobs.thr ? 1 : 0;
        }
    }
}

// UPDATE = false: dw += lambda * d(penalty)/dw.   UPDATE = true: the optimizer step with the regulariser folded in,
//   g = dw + wd*w + lambda*w*(a/out_norm + b/in_norm);  mom = mu*mom + g;  w -= lr*mom   (one pass over w, dw, mom).
struct StepParams {
    float lr, mu, wd;
};
template <int VEC, bool UPDATE>
__global__ __launch_bounds__(kThreads) void k_group_lasso_grad(const LassoJobs jobs, float lambda, StepParams sp) {
    const int ji = find_job(jobs, blockIdx.x);
    const LassoJob& J = jobs.j[ji];
    const int chunk = blockIdx.x - J.first_block;
    const int tid = threadIdx.x;
    const int TX = 1 << J.txlog2, TY = kThreads >> J.txlog2;
    const int tx = tid & (TX - 1), ty = tid >> J.txlog2;
    const int C = J.C, cpitch = J.cpitch, RS = J.RS;
    const int Lv = (C + VEC - 1) / VEC;
    const int64_t rows = (int64_t)J.K * RS;
    const int64_t r0 = (int64_t)chunk * J.rows_per_chunk;
    const int64_t r1 = min(rows, r0 + J.rows_per_chunk);
    const bool reg_out = J.flags & PT_LASSO_OUT, reg_in = J.flags & PT_LASSO_IN;
    float* __restrict__ w = const_cast<float*>(J.w);
    float* __restrict__ dw = J.dw;
    float* __restrict__ mom = J.mom;

    for (int cg = tx; cg < Lv; cg += TX) {
        float inv_in[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const int c = cg * VEC + e;
            const float nrm = (reg_in && c < C) ? J.in_norm[c] : 0.f;
            inv_in[e] = nrm > 0.f ? 1.0f / nrm : 0.f;
        }
#pragma unroll 4
        for (int64_t r = r0 + ty; r < r1; r += TY) {
            const int k = (int)(r / RS);
            const float on = reg_out ? J.out_norm[k] : 0.f;
            const float inv_out = on > 0.f ? 1.0f / on : 0.f;
            const size_t off = (size_t)r * cpitch + (size_t)cg * VEC;
            float v[VEC], g[VEC];
            load_vec<VEC>(w + off, v);
            load_vec<VEC>(dw + off, g);
#pragma unroll
            for (int e = 0; e < VEC; ++e) g[e] += lambda * (v[e] * (inv_out + inv_in[e]));
            float* dst = dw;
            if constexpr (UPDATE) {
                float m[VEC];
                load_vec<VEC>(mom + off, m);
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    m[e] = sp.mu * m[e] + (g[e] + sp.wd * v[e]);
                    g[e] = v[e] - sp.lr * m[e];  // g now holds the new weight
                }
                if constexpr (VEC == 4) {
                    if (cg * 4 + 3 < C) {
                        *reinterpret_cast<float4*>(mom + off) = make_float4(m[0], m[1], m[2], m[3]);
                    } else {
                        for (int e = 0; e < 4; ++e)
                            if (cg * 4 + e < C) mom[off + e] = m[e];
                    }
                } else {
                    mom[off] = m[0];
                }
                dst = w;
            }
            if constexpr (VEC == 4) {
                if (cg * 4 + 3 < C) {
                    *reinterpret_cast<float4*>(dst + off) = make_float4(g[0], g[1], g[2], g[3]);
                } else {
                    for (int e = 0; e < 4; ++e)
                        if (cg * 4 + e < C) dst[off + e] = g[e];
                }
            } else {
                dst[off] = g[0];
            }
        }
    }
}

// ---- host-side planning ---------------------------------------------------------------------- //
struct ChunkPlan {
    int txlog2, rows_per_chunk, n_chunks;
};

// Gradient / optimizer pass and the element-wise norms pass: TX lanes across a row, about 16 K elements per workgroup.
static ChunkPlan plan_chunks(int64_t rows, int C, bool vec) {
    const int Lv = vec ? (C + 3) / 4 : C;
    int l = 0;
    while ((1 << l) < Lv && l < 6) ++l;
    const int TY = kThreads >> l;
    int64_t rpc = ceil_div(16384, C);
    rpc = round_up(rpc, TY);
    ChunkPlan p;
    p.txlog2 = l;
    p.rows_per_chunk = (int)rpc;
    p.n_chunks = (int)ceil_div(rows, rpc);
    return p;
}

// Vector norms pass: a workgroup streams whole batches of TY * U rows (256 threads x eight 16-byte loads, 8 K
// elements when every lane has a column), kNormBatches of them per chunk.
constexpr int kNormBatches = 2;
static ChunkPlan plan_norm_chunks(int64_t rows, int C) {
    const NormLayout l = norm_layout(C);
    const int batch_rows = (kThreads >> l.txlog2) * (8 >> l.cglog2);
    ChunkPlan p;
    p.txlog2 = l.txlog2;
    p.rows_per_chunk = batch_rows * kNormBatches;
    p.n_chunks = (int)ceil_div(rows, p.rows_per_chunk);
    return p;
}

static bool norms_vec_ok(const NormLayer& L) {
    return (L.cpitch % 4 == 0) && (((uintptr_t)L.w & 15) == 0) && (!L.shadow || ((uintptr_t)L.shadow & 7) == 0) && L.C <= kMaxC;
}

int32_t check_norm_layer(const NormLayer& L) {
    if (!L.w || !L.out_norm || !L.in_norm) return PT_ERR_NULL;
    if (L.K <= 0 || L.RS <= 0 || L.C <= 0 || L.cpitch < L.C) return PT_ERR_SHAPE;
    if (L.C > kMaxC) return PT_ERR_UNSUPPORTED;  // register tile of the column sums
    if ((int64_t)L.K * L.RS >= (1ll << 31)) return PT_ERR_UNSUPPORTED;
    return PT_OK;
}

// Workspace of one layer: row sums + per-chunk column partials, sized for whichever loader is used.
size_t norm_layer_ws_bytes(int32_t K, int32_t RS, int32_t C) {
    const int64_t rows = (int64_t)K * RS;
    const ChunkPlan a = plan_norm_chunks(rows, C), b = plan_chunks(rows, C, false);
    const int n_chunks = a.n_chunks > b.n_chunks ? a.n_chunks : b.n_chunks;
    return (size_t)round_up((rows + (int64_t)n_chunks * C) * 4, 256);
}

// Group norms (and optionally zero masks) of n layers: one partial + one finish launch per kMaxJobs layers of a
// loader kind.  The workspace is split between the layers in array order.
int32_t launch_norms(const NormLayer* layers, int n, void* ws, size_t ws_bytes, float thr, hipStream_t st) {
    size_t need = 0;
    for (int i = 0; i < n; ++i) {
        const int32_t rc = check_norm_layer(layers[i]);
        if (rc != PT_OK) return rc;
        need += norm_layer_ws_bytes(layers[i].K, layers[i].RS, layers[i].C);
    }
    if (!ws) return PT_ERR_NULL;
    if (ws_bytes < need) return PT_ERR_WORKSPACE;
    if (((uintptr_t)ws & 15) != 0) return PT_ERR_SHAPE;
    if (need / 4 >= (1ull << 32)) return PT_ERR_UNSUPPORTED;
    for (int pass = 0; pass < 2; ++pass) {
        const bool want_vec = pass == 0;
        NormJobs jobs;
        jobs.n = 0;
        jobs.ws = (float*)ws;
        jobs.thr = thr;
        int64_t blocks = 0, fin_blocks = 0;
        auto flush = [&]() -> int32_t {
            if (jobs.n == 0) return PT_OK;
            if (want_vec) hipLaunchKernelGGL(k_group_norms_partial_vec, dim3((unsigned)blocks), dim3(kThreads), 0, st, jobs);
            else hipLaunchKernelGGL(k_group_norms_partial_elem, dim3((unsigned)blocks), dim3(kThreads), 0, st, jobs);
            int32_t rc = launch_status();
            if (rc != PT_OK) return rc;
            hipLaunchKernelGGL(k_group_norms_finish, dim3((unsigned)fin_blocks), dim3(kThreads), 0, st, jobs);
            jobs.n = 0;
            blocks = 0;
            fin_blocks = 0;
            return launch_status();
        };
        size_t off = 0;  // bytes
        for (int i = 0; i < n; ++i) {
            const NormLayer& L = layers[i];
            const size_t bytes = norm_layer_ws_bytes(L.K, L.RS, L.C);
            if (norms_vec_ok(L) == want_vec) {
                const int64_t rows = (int64_t)L.K * L.RS;
                const ChunkPlan cp = want_vec ? plan_norm_chunks(rows, L.C) : plan_chunks(rows, L.C, false);
                if (blocks + cp.n_chunks > 0x3fffffff) {
                    const int32_t rc = flush();
                    if (rc != PT_OK) return rc;
                }
                NormJob& J = jobs.j[jobs.n++];
                J.w = L.w; J.shadow = L.shadow; J.out_norm = L.out_norm; J.in_norm = L.in_norm;
                J.zero_out = L.zero_out; J.zero_in = L.zero_in;
                J.ws_off = (uint32_t)(off / 4);
                J.K = L.K; J.RS = L.RS; J.C = L.C; J.cpitch = L.cpitch;
                J.first_block = (int)blocks; J.n_chunks = cp.n_chunks; J.rows_per_chunk = cp.rows_per_chunk;
                J.fin_first = (int)fin_blocks;
                blocks += cp.n_chunks;
                fin_blocks += ceil_div((int64_t)L.K + L.C, kFinGroups);
                if (jobs.n == kMaxJobs) {
                    const int32_t rc = flush();
                    if (rc != PT_OK) return rc;
                }
            }
            off += bytes;
        }
        const int32_t rc = flush();
        if (rc != PT_OK) return rc;
    }
    return PT_OK;
}

// Value of the regulariser (GroupLassoReg of Alg. 1): the sum of the enabled group norms of up to
// kMaxPenaltyJobs layers, ONE workgroup, fp64 accumulation in a fixed order (thread t adds elements
// t, t+1024, ... of the concatenated norm vectors; a fixed tree adds the 1024 thread sums), so the value is
// run-to-run identical.  A few 10^4 floats: the launch's fixed cost is all of it.
constexpr int kMaxPenaltyJobs = 96;
struct PenaltyJob {
    const float* out_norm;
    const float* in_norm;
    int K, C;  // 0 when that group kind is not regularised
};
struct PenaltyJobs {
    PenaltyJob j[kMaxPenaltyJobs];
    int n, accumulate;
};
__global__ __launch_bounds__(1024) void k_group_lasso_penalty(const PenaltyJobs jobs, double* __restrict__ penalty) {
    __shared__ double red[1024];
    const int tid = threadIdx.x;
    double s = 0.0;
    int base = 0;  // position of the current vector in the concatenation, modulo 1024
    for (int i = 0; i < jobs.n; ++i) {
        const PenaltyJob& J = jobs.j[i];
        for (int v = 0; v < 2; ++v) {
            const float* p = v == 0 ? J.out_norm : J.in_norm;
            const int n = v == 0 ? J.K : J.C;
            // element e of this vector belongs to thread (base + e) % 1024
            for (int e = (tid - base + 1024) & 1023; e < n; e += 1024) s += (double)p[e];
            base = (base + n) & 1023;
        }
    }
    red[tid] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if (tid < w) red[tid] += red[tid + w];
        __syncthreads();
    }
    if (tid == 0) *penalty = (jobs.accumulate ? *penalty : 0.0) + red[0];
}

}  // namespace pt

using namespace pt;

extern "C" int32_t pt_group_norms_batched_workspace_bytes(const pt_layer_weights* layers, int32_t n, size_t* bytes) {
    if (!bytes || (n > 0 && !layers)) return PT_ERR_NULL;
    if (n < 0) return PT_ERR_SHAPE;
    size_t total = 0;
    for (int i = 0; i < n; ++i) {
        if (layers[i].K <= 0 || layers[i].RS <= 0 || layers[i].C <= 0) return PT_ERR_SHAPE;
        total += norm_layer_ws_bytes(layers[i].K, layers[i].RS, layers[i].C);
    }
    *bytes = total;
    return PT_OK;
}

extern "C" int32_t pt_group_norms_batched(const pt_layer_weights* layers, int32_t n, void* ws, size_t ws_bytes,
                                          void* stream) {
    if (n < 0) return PT_ERR_SHAPE;
    if (n == 0) return PT_OK;
    if (!layers || !ws) return PT_ERR_NULL;
    std::vector<NormLayer> v((size_t)n);
    for (int i = 0; i < n; ++i) {
        const pt_layer_weights& L = layers[i];
        v[i] = NormLayer{L.w, L.out_norm, L.in_norm, L.w_shadow, nullptr, nullptr, L.K, L.RS, L.C, L.w_cpitch};
    }
    return launch_norms(v.data(), n, ws, ws_bytes, 0.f, (hipStream_t)stream);
}

extern "C" int32_t pt_group_norms_detect_batched_workspace_bytes(const pt_layer_detect* layers, int32_t n, size_t* bytes) {
    if (!bytes || (n > 0 && !layers)) return PT_ERR_NULL;
    if (n < 0) return PT_ERR_SHAPE;
    size_t total = 0;
    for (int i = 0; i < n; ++i) {
        if (layers[i].K <= 0 || layers[i].RS <= 0 || layers[i].C <= 0) return PT_ERR_SHAPE;
        total += norm_layer_ws_bytes(layers[i].K, layers[i].RS, layers[i].C);
    }
    *bytes = total;
    return PT_OK;
}

extern "C" int32_t pt_group_norms_detect_batched(const pt_layer_detect* layers, int32_t n, float thr, void* ws,
                                                 size_t ws_bytes, void* stream) {
    if (n < 0) return PT_ERR_SHAPE;
    if (n == 0) return PT_OK;
    if (!layers || !ws) return PT_ERR_NULL;
    std::vector<NormLayer> v((size_t)n);
    for (int i = 0; i < n; ++i) {
        const pt_layer_detect& L = layers[i];
        if (!L.zero_out || !L.zero_in) return PT_ERR_NULL;
        v[i] = NormLayer{L.w, L.out_norm, L.in_norm, nullptr, L.zero_out, L.zero_in, L.K, L.RS, L.C, L.w_cpitch};
    }
    return launch_norms(v.data(), n, ws, ws_bytes, thr, (hipStream_t)stream);
}

// Shared launcher of the gradient pass and of the optimizer step (mom == nullptr in every layer <=> gradient pass).
struct LassoLayer {
    const float* w;
    const float* out_norm;
    const float* in_norm;
    float* dw;
    float* mom;
    int32_t K, RS, C, w_cpitch;
    uint32_t flags;
};
static int32_t launch_lasso(const LassoLayer* layers, int n, bool update, float lambda, StepParams sp, hipStream_t st) {
    for (int pass = 0; pass < 2; ++pass) {
        const bool want_vec = pass == 0;
        LassoJobs jobs;
        jobs.n = 0;
        int blocks = 0;
        auto flush = [&]() -> int32_t {
            if (jobs.n == 0) return PT_OK;
            if (want_vec && update)
                hipLaunchKernelGGL((k_group_lasso_grad<4, true>), dim3(blocks), dim3(kThreads), 0, st, jobs, lambda, sp);
            else if (want_vec)
                hipLaunchKernelGGL((k_group_lasso_grad<4, false>), dim3(blocks), dim3(kThreads), 0, st, jobs, lambda, sp);
            else if (update)
                hipLaunchKernelGGL((k_group_lasso_grad<1, true>), dim3(blocks), dim3(kThreads), 0, st, jobs, lambda, sp);
            else
                hipLaunchKernelGGL((k_group_lasso_grad<1, false>), dim3(blocks), dim3(kThreads), 0, st, jobs, lambda, sp);
            jobs.n = 0;
            blocks = 0;
            return launch_status();
        };
        for (int i = 0; i < n; ++i) {
            const LassoLayer& L = layers[i];
            const bool vec = (L.w_cpitch % 4 == 0) && (((uintptr_t)L.w & 15) == 0) && (((uintptr_t)L.dw & 15) == 0) &&
                             (!update || ((uintptr_t)L.mom & 15) == 0);
            if (vec != want_vec) continue;
            const ChunkPlan cp = plan_chunks((int64_t)L.K * L.RS, L.C, vec);
            LassoJob& J = jobs.j[jobs.n++];
            J.w = L.w; J.out_norm = L.out_norm; J.in_norm = L.in_norm; J.dw = L.dw; J.mom = L.mom;
            J.K = L.K; J.RS = L.RS; J.C = L.C; J.cpitch = L.w_cpitch;
            J.first_block = blocks; J.n_chunks = cp.n_chunks; J.rows_per_chunk = cp.rows_per_chunk; J.txlog2 = cp.txlog2;
            J.flags = L.flags; J.pad = 0;
            blocks += cp.n_chunks;
            if (jobs.n == kMaxLassoJobs) {
                int32_t rc = flush();
                if (rc != PT_OK) return rc;
            }
        }
        int32_t rc = flush();
        if (rc != PT_OK) return rc;
    }
    return PT_OK;
}

extern "C" int32_t pt_group_lasso_grad_batched(const pt_layer_lasso* layers, int32_t n, float lambda, void* stream) {
    if (n < 0) return PT_ERR_SHAPE;
    if (n == 0) return PT_OK;
    if (!layers) return PT_ERR_NULL;
    for (int i = 0; i < n; ++i) {
        const pt_layer_lasso& L = layers[i];
        if (!L.w || !L.out_norm || !L.in_norm || !L.dw) return PT_ERR_NULL;
        if (L.K <= 0 || L.RS <= 0 || L.C <= 0 || L.w_cpitch < L.C) return PT_ERR_SHAPE;
        if (L.flags & ~3u) return PT_ERR_UNSUPPORTED;
    }
    std::vector<LassoLayer> v((size_t)n);
    for (int i = 0; i < n; ++i) {
        const pt_layer_lasso& L = layers[i];
        v[i] = LassoLayer{L.w, L.out_norm, L.in_norm, L.dw, nullptr, L.K, L.RS, L.C, L.w_cpitch, L.flags};
    }
    return launch_lasso(v.data(), n, false, lambda, StepParams{0.f, 0.f, 0.f}, (hipStream_t)stream);
}

extern "C" int32_t pt_sgd_momentum_lasso_batched(const pt_layer_update* layers, int32_t n, float lambda, float lr,
                                                 float momentum, float weight_decay, void* stream) {
    if (n < 0) return PT_ERR_SHAPE;
    if (n == 0) return PT_OK;
    if (!layers) return PT_ERR_NULL;
    for (int i = 0; i < n; ++i) {
        const pt_layer_update& L = layers[i];
        if (!L.w || !L.dw || !L.mom || !L.out_norm || !L.in_norm) return PT_ERR_NULL;
        if (L.K <= 0 || L.RS <= 0 || L.C <= 0 || L.w_cpitch < L.C) return PT_ERR_SHAPE;
        if (L.flags & ~3u) return PT_ERR_UNSUPPORTED;
    }
    std::vector<LassoLayer> v((size_t)n);
    for (int i = 0; i < n; ++i) {
        const pt_layer_update& L = layers[i];
        v[i] = LassoLayer{L.w, L.out_norm, L.in_norm, const_cast<float*>(L.dw), L.mom, L.K, L.RS, L.C, L.w_cpitch, L.flags};
    }
    return launch_lasso(v.data(), n, true, lambda, StepParams{lr, momentum, weight_decay}, (hipStream_t)stream);
}

// ---- single-layer forms: the batched calls with one entry ------------------------------------- //
extern "C" int32_t pt_group_norms_workspace_bytes(int32_t K, int32_t RS, int32_t C, size_t* bytes) {
    if (!bytes) return PT_ERR_NULL;
    if (K <= 0 || RS <= 0 || C <= 0) return PT_ERR_SHAPE;
    *bytes = norm_layer_ws_bytes(K, RS, C);
    return PT_OK;
}

extern "C" int32_t pt_group_norms(const float* w, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch, float* out_norm,
                                  float* in_norm, uint16_t* w_shadow, void* ws, size_t ws_bytes, void* stream) {
    if (!w || !out_norm || !in_norm || !ws) return PT_ERR_NULL;
    pt_layer_weights L{};
    L.w = w; L.K = K; L.RS = RS; L.C = C; L.w_cpitch = w_cpitch;
    L.out_norm = out_norm; L.in_norm = in_norm; L.w_shadow = w_shadow;
    return pt_group_norms_batched(&L, 1, ws, ws_bytes, stream);
}

extern "C" int32_t pt_group_lasso_grad(const float* w, const float* out_norm, const float* in_norm, float lambda,
                                       uint32_t flags, float* dw, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch,
                                       void* stream) {
    pt_layer_lasso L{};
    L.w = w; L.out_norm = out_norm; L.in_norm = in_norm; L.dw = dw;
    L.K = K; L.RS = RS; L.C = C; L.w_cpitch = w_cpitch; L.flags = flags;
    return pt_group_lasso_grad_batched(&L, 1, lambda, stream);
}

extern "C" int32_t pt_group_lasso_penalty_batched(const pt_layer_penalty* layers, int32_t n, double* penalty_dev,
                                                  void* stream) {
    if (n < 0) return PT_ERR_SHAPE;
    if (!penalty_dev || (n > 0 && !layers)) return PT_ERR_NULL;
    for (int i = 0; i < n; ++i) {
        if (layers[i].K < 0 || layers[i].C < 0) return PT_ERR_SHAPE;
        if (layers[i].flags & ~(PT_LASSO_OUT | PT_LASSO_IN)) return PT_ERR_UNSUPPORTED;
        if (((layers[i].flags & PT_LASSO_OUT) && layers[i].K > 0 && !layers[i].out_norm) ||
            ((layers[i].flags & PT_LASSO_IN) && layers[i].C > 0 && !layers[i].in_norm))
            return PT_ERR_NULL;
    }
    PenaltyJobs jobs;
    jobs.n = 0;
    jobs.accumulate = 0;
    int i = 0;
    do {  // at least one launch, so that n == 0 writes 0
        for (; i < n && jobs.n < kMaxPenaltyJobs; ++i) {
            const pt_layer_penalty& L = layers[i];
            jobs.j[jobs.n++] = PenaltyJob{L.out_norm, L.in_norm, (L.flags & PT_LASSO_OUT) ? L.K : 0,
                                          (L.flags & PT_LASSO_IN) ? L.C : 0};
        }
        hipLaunchKernelGGL(k_group_lasso_penalty, dim3(1), dim3(1024), 0, (hipStream_t)stream, jobs, penalty_dev);
        const int32_t rc = launch_status();
        if (rc != PT_OK) return rc;
        jobs.n = 0;
        jobs.accumulate = 1;
    } while (i < n);
    return PT_OK;
}

extern "C" int32_t pt_lasso_set_coeff(double loss1, double loss2, double ratio, double* lambda) {
    if (!lambda) return PT_ERR_NULL;
    if (!(ratio > 0.0 && ratio < 1.0) || !(loss2 > 0.0) || !(loss1 >= 0.0)) return PT_ERR_SHAPE;
    *lambda = ratio * loss1 / ((1.0 - ratio) * loss2);
    return PT_OK;
}
