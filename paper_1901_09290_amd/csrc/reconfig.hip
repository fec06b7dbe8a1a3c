// Reconfiguration kernels (Sec. 4.1-4.2): zero-group detection, channel-edge reconciliation,
// compaction plan (prefix sum over the keep mask) and the compaction gathers.  All integer/byte
// results are exact; the gathers are pure data movement and HBM-bound.
#include "common.h"

namespace pt {

__global__ void k_zero_groups(const float* __restrict__ norms, int n, float thr, uint8_t* __restrict__ zero) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) zero[i] = norms[i] < thr ? 1 : 0;
}

constexpr int kMaxEdgeMembers = 64;
struct EdgeMasks {
    const uint8_t* m[kMaxEdgeMembers];
    int count;
};

// keep[j] = 0 iff channel j is flagged zero by every member of the edge.
__global__ void k_reconcile_edge(EdgeMasks e, int n, uint8_t* __restrict__ keep) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n) return;
    uint8_t all_zero = 1;
    for (int a = 0; a < e.count; ++a) all_zero &= (e.m[a][j] != 0);
    keep[j] = all_zero ? 0 : 1;
}

// Single workgroup, 1024 threads: chunked exclusive scan with wavefront ballots.
__global__ __launch_bounds__(1024) void k_compact_plan(const uint8_t* __restrict__ keep, int n, int* __restrict__ idx,
                                                       int* __restrict__ n_keep) {
    __shared__ int wave_tot[16];
    __shared__ int base_s;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) base_s = 0;
    __syncthreads();
    for (int j0 = 0; j0 < n; j0 += 1024) {
        const int j = j0 + tid;
        const bool k = (j < n) && keep[j] != 0;
        const unsigned long long b = __ballot(k);
        const int pre = __popcll(b & ((1ull << lane) - 1ull));
        if (lane == 0) wave_tot[wv] = __popcll(b);
        __syncthreads();
        int off = base_s;
        for (int a = 0; a < wv; ++a) off += wave_tot[a];
        if (k) idx[off + pre] = j;
        __syncthreads();
        if (tid == 0) {
            int t = 0;
            for (int a = 0; a < 16; ++a) t += wave_tot[a];
            base_s += t;
        }
        __syncthreads();
    }
    if (tid == 0) *n_keep = base_s;
}

// One thread per output element group of 4 consecutive c'.
__global__ void k_compact_weights(const float* __restrict__ w, int RS, int cpitch, const int* __restrict__ idxK,
                                  const int* __restrict__ idxC, int Cp, int out_cpitch, int64_t out_rows,
                                  float* __restrict__ out) {
    const int cq = (Cp + 3) >> 2;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= out_rows * cq) return;
    const int64_t row = t / cq;          // k' * RS + rs
    const int c0 = (int)(t - row * cq) * 4;
    const int64_t kp = row / RS;
    const int rs = (int)(row - kp * RS);
    const int64_t k = idxK ? idxK[kp] : kp;
    const float* src = w + (k * RS + rs) * (int64_t)cpitch;
    float* dst = out + row * (int64_t)out_cpitch + c0;
    float v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int c = c0 + e;
        v[e] = (c < Cp) ? src[idxC ? idxC[c] : c] : 0.f;
    }
    if (c0 + 3 < Cp && (out_cpitch & 3) == 0 && (((uintptr_t)out & 15) == 0)) {
        *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (c0 + e < Cp) dst[e] = v[e];
    }
}

template <typename T>
__global__ void k_compact_vector(const T* __restrict__ v, const int* __restrict__ idx, int n_keep, T* __restrict__ out) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < n_keep) out[j] = v[idx[j]];
}

// Activation gather along the innermost axis, element-wise form (any pitch / alignment): one thread
// produces 8 consecutive output channels of one pixel.  Padding channels of the last group of eight that lie
// inside the row are written as zero (rows are then written without holes wherever the pitch allows it).
__global__ void k_compact_nhwc(const uint16_t* __restrict__ x, int64_t pixels, int x_cpitch,
                               const int* __restrict__ idx, int Cp, uint16_t* __restrict__ out, int out_cpitch,
                               int vec_ok) {
    const int cv = (Cp + 7) >> 3;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= pixels * cv) return;
    const int64_t pix = t / cv;
    const int c0 = (int)(t - pix * cv) * 8;
    const uint16_t* src = x + pix * (int64_t)x_cpitch;
    uint16_t* dst = out + pix * (int64_t)out_cpitch + c0;
    uint16_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (c0 + e < Cp) ? src[idx[c0 + e]] : (uint16_t)0;
    if (vec_ok) {  // pitch a multiple of 8: the whole group lies inside the row
        uint4 o;
        o.x = v[0] | ((uint32_t)v[1] << 16);
        o.y = v[2] | ((uint32_t)v[3] << 16);
        o.z = v[4] | ((uint32_t)v[5] << 16);
        o.w = v[6] | ((uint32_t)v[7] << 16);
        *reinterpret_cast<uint4*>(dst) = o;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (c0 + e < out_cpitch) dst[e] = v[e];
    }
}

// Activation gather, streaming form (16-byte aligned rows on both sides).  A workgroup streams runs of whole
// pixel rows through two LDS buffers with direct global->LDS loads (every source byte is read once, fully
// coalesced, and the next run is in flight while the current one is gathered); every thread keeps its eight
// channel indices in registers, assembles 8 output channels of a pixel from LDS with eight 16-bit reads and
// writes one 16-byte store.  Channels of the last vector past Cp are written as zero: rows without holes keep
// the memory system from merging partial lines (measured: stores of ragged rows with holes ran at half the
// rate of whole rows).
constexpr int kGatherThreads = 256;
constexpr int kGatherChunk = 32 * 1024;                           // bytes of pixel rows per LDS buffer
constexpr int kGatherLoads = kGatherChunk / (kGatherThreads * 16);  // 16-byte loads per thread and run (8)
typedef __attribute__((address_space(3))) void* lds_vptr;
typedef const __attribute__((address_space(1))) void* glb_vptr;

// Up to kMaxGatherJobs activation tensors per launch: runs ("chunks") of all tensors form one global sequence
// that the workgroups walk with a fixed stride; a workgroup re-reads its eight channel indices only when the
// tensor changes between two of its runs.
constexpr int kMaxGatherJobs = 64;
struct GatherJob {
    const uint16_t* x;
    const int* idx;
    uint16_t* out;
    int64_t pixels;
    int x_cpitch, Cp, out_cpitch, ppc;  // ppc: pixels per run
    int chunk0, pad;                    // first run of this tensor in the global sequence
};
struct GatherJobs {
    GatherJob j[kMaxGatherJobs];
    int n, total_chunks;
};

__global__ __launch_bounds__(kGatherThreads) void k_compact_nhwc_lds(const GatherJobs jobs) {
#if defined(__HIP_DEVICE_COMPILE__)
    extern __shared__ __attribute__((aligned(16))) uint8_t sbuf[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_vptr)sbuf;
    const int total = jobs.total_chunks;

    auto job_of = [&](int g) {  // last job whose chunk0 <= g (uniform)
        int lo = 0, hi = jobs.n - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (jobs.j[mid].chunk0 <= g) lo = mid;
            else hi = mid - 1;
        }
        return lo;
    };
    // Every wave issues exactly kGatherLoads load instructions per run (lanes past the run's end re-read its last
    // 16 bytes into a slot nobody reads), so "at most kGatherLoads outstanding" means the previous run has landed.
    auto issue = [&](int g, int buf) {
        const GatherJob& J = jobs.j[job_of(g)];
        const int64_t p0 = (int64_t)(g - J.chunk0) * J.ppc;
        const int np = (int)min((int64_t)J.ppc, J.pixels - p0);
        const int n16 = np * (J.x_cpitch >> 3);
        const uint8_t* src = reinterpret_cast<const uint8_t*>(J.x + p0 * J.x_cpitch);
#pragma unroll
        for (int k = 0; k < kGatherLoads; ++k) {
            const int i0 = k * kGatherThreads + wave * 64;
            const int i = min(i0 + lane, n16 - 1);
            __builtin_amdgcn_global_load_lds((glb_vptr)(uintptr_t)(src + (size_t)i * 16),
                                             (lds_vptr)(sbuf + buf * kGatherChunk + i0 * 16), 16, 0, 0);
        }
    };

    // gather-side state of the current tensor
    int cur = -1, ppb = 1, pp = 0, v = 0, row_bytes = 0;
    uint32_t m0 = 0, m1 = 0, m2 = 0, m3 = 0;   // which halves of the four output words hold channels < Cp
    bool active = false;
    uint32_t id2[8] = {0, 0, 0, 0, 0, 0, 0, 0};  // byte offset of each source channel inside a pixel row

    int g = blockIdx.x;
    if (g < total) issue(g, 0);
    for (int it = 0; g < total; g += gridDim.x, ++it) {
        const int buf = it & 1;
        const bool more = g + (int)gridDim.x < total;
        if (more) {
            issue(g + gridDim.x, buf ^ 1);
            __builtin_amdgcn_s_waitcnt((kGatherLoads & 15) | (7 << 4) | (15 << 8) | ((kGatherLoads >> 4) << 14));
        } else {
            __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();            // this run has landed for every wave
        asm volatile("" ::: "memory");
        const int ji = job_of(g);
        const GatherJob& J = jobs.j[ji];
        if (ji != cur) {                         // uniform: a new tensor, new thread roles and channel indices
            cur = ji;
            const int nvec = (J.Cp + 7) >> 3;
            ppb = kGatherThreads / nvec;         // pixels gathered per pass (nvec <= 256)
            pp = tid / nvec;
            v = tid - pp * nvec;
            active = pp < ppb;
#pragma unroll
            for (int e = 0; e < 8; ++e) id2[e] = (active && v * 8 + e < J.Cp) ? 2u * (uint32_t)J.idx[v * 8 + e] : 0u;
            const int nlast = J.Cp - v * 8;      // valid channels of this thread's vector (>= 8: all)
            auto halves = [&](int k) { return (k < nlast ? 0xFFFFu : 0u) | (k + 1 < nlast ? 0xFFFF0000u : 0u); };
            m0 = halves(0); m1 = halves(2); m2 = halves(4); m3 = halves(6);
            row_bytes = J.x_cpitch * 2;
        }
        const int64_t p0 = (int64_t)(g - J.chunk0) * J.ppc;
        const int np = (int)min((int64_t)J.ppc, J.pixels - p0);
        if (active) {
            for (int p = pp; p < np; p += ppb) {
                const uint32_t r = lds_base + (uint32_t)(buf * kGatherChunk + p * row_bytes);
                uint32_t e[8];
                // 16-bit LDS reads issued back to back; one wait, then pairs are packed into the output registers
#pragma unroll
                for (int k = 0; k < 8; ++k) asm volatile("ds_read_u16 %0, %1" : "=v"(e[k]) : "v"(r + id2[k]));
                asm volatile("s_waitcnt lgkmcnt(0)"
                             : "+v"(e[0]), "+v"(e[1]), "+v"(e[2]), "+v"(e[3]), "+v"(e[4]), "+v"(e[5]), "+v"(e[6]), "+v"(e[7]));
                const uint32_t o0 = (e[0] | (e[1] << 16)) & m0, o1 = (e[2] | (e[3] << 16)) & m1;
                const uint32_t o2 = (e[4] | (e[5] << 16)) & m2, o3 = (e[6] | (e[7] << 16)) & m3;
                uint16_t* dst = J.out + (p0 + p) * (int64_t)J.out_cpitch + v * 8;
                *reinterpret_cast<uint4*>(dst) = make_uint4(o0, o1, o2, o3);
            }
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();            // everyone is done with this buffer before it is refilled
        asm volatile("" ::: "memory");
    }
#endif
}

// ---- multi-job forms: a network has dozens of layers and edges and each of these steps is tiny, so the job
// descriptors ride in the kernel arguments of one launch and a workgroup looks up which job it serves.
constexpr int kMaxMaskJobs = 128;
struct MaskJob {
    const float* norms;
    uint8_t* zero;
    int n, blk0;  // blk0: first workgroup of this job
};
struct MaskJobs {
    MaskJob j[kMaxMaskJobs];
    int n;
};
template <typename Jobs>
__device__ __forceinline__ int job_of_block(const Jobs& jobs, int block) {
    int lo = 0, hi = jobs.n - 1;  // last job whose blk0 <= block
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs.j[mid].blk0 <= block) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}
__global__ __launch_bounds__(256) void k_zero_groups_multi(const MaskJobs jobs, float thr) {
    const int ji = job_of_block(jobs, blockIdx.x);
    const MaskJob& jb = jobs.j[ji];
    const int i = (blockIdx.x - jb.blk0) * 256 + threadIdx.x;
    if (i < jb.n) jb.zero[i] = jb.norms[i] < thr ? 1 : 0;
}

// One workgroup per edge: keep mask from the members' zero masks, then the ascending survivor list by a
// chunked exclusive scan (wavefront ballots), all inside the workgroup.
constexpr int kMaxPlanEdges = 64, kMaxPlanMembers = 320;  // 5 KB of kernel arguments: a ResNet-50 (37 edges) is one launch
struct PlanEdge {
    uint8_t* keep;
    int* idx;
    int* n_keep;
    int n, m0, mcount;  // members m[m0 .. m0+mcount)
};
struct PlanJobs {
    PlanEdge e[kMaxPlanEdges];
    const uint8_t* m[kMaxPlanMembers];
};
__global__ __launch_bounds__(1024) void k_reconcile_plan_multi(const PlanJobs jobs) {
    __shared__ int wave_tot[16];
    __shared__ int base_s;
    const PlanEdge& e = jobs.e[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) base_s = 0;
    __syncthreads();
    for (int j0 = 0; j0 < e.n; j0 += 1024) {
        const int j = j0 + tid;
        bool k = false;
        if (j < e.n) {
            uint8_t all_zero = 1;
            for (int a = 0; a < e.mcount; ++a) all_zero &= (jobs.m[e.m0 + a][j] != 0);
            k = !all_zero;
            e.keep[j] = k ? 1 : 0;
        }
        const unsigned long long b = __ballot(k);
        const int pre = __popcll(b & ((1ull << lane) - 1ull));
        if (lane == 0) wave_tot[wv] = __popcll(b);
        __syncthreads();
        int off = base_s;
        for (int a = 0; a < wv; ++a) off += wave_tot[a];
        if (k) e.idx[off + pre] = j;
        __syncthreads();
        if (tid == 0) {
            int t = 0;
            for (int a = 0; a < 16; ++a) t += wave_tot[a];
            base_s += t;
        }
        __syncthreads();
    }
    if (tid == 0) *e.n_keep = base_s;
}

constexpr int kMaxVecJobs = 224;  // 9 KB of kernel arguments: four vectors for each of 53 layers in one launch
struct VecJob {
    const void* v;
    const int* idx;
    void* out;
    int n_keep, elem_bytes, blk0, pad;
};
struct VecJobs {
    VecJob j[kMaxVecJobs];
    int n;
};
__global__ __launch_bounds__(256) void k_compact_vector_multi(const VecJobs jobs) {
    const int ji = job_of_block(jobs, blockIdx.x);
    const VecJob& jb = jobs.j[ji];
    const int t = (blockIdx.x - jb.blk0) * 256 + threadIdx.x;
    if (t >= jb.n_keep) return;
    const int s = jb.idx[t];
    switch (jb.elem_bytes) {
        case 1: ((uint8_t*)jb.out)[t] = ((const uint8_t*)jb.v)[s]; break;
        case 2: ((uint16_t*)jb.out)[t] = ((const uint16_t*)jb.v)[s]; break;
        case 4: ((uint32_t*)jb.out)[t] = ((const uint32_t*)jb.v)[s]; break;
        default: ((uint64_t*)jb.out)[t] = ((const uint64_t*)jb.v)[s]; break;
    }
}

constexpr int kMaxWJobs = 112;  // 7 KB of kernel arguments: weights and momentum of 53 layers in one launch
struct WJob {
    const float* w;
    const int* idxK;
    const int* idxC;
    float* out;
    int RS, cpitch, Cp, out_cpitch, out_rows, blk0, rows_per_blk, pad;
};
struct WJobs {
    WJob j[kMaxWJobs];
    int n;
};
// A workgroup gathers `rows_per_blk` consecutive output rows (k', rs) of one tensor; a thread produces 4
// consecutive c' of a row.
__global__ __launch_bounds__(256) void k_compact_weights_multi(const WJobs jobs) {
    const int ji = job_of_block(jobs, blockIdx.x);
    const WJob& jb = jobs.j[ji];
    const int cq = (jb.Cp + 3) >> 2;
    const int row0 = (blockIdx.x - jb.blk0) * jb.rows_per_blk;
    const int nrow = min(jb.rows_per_blk, jb.out_rows - row0);
    const bool vec = (jb.out_cpitch & 3) == 0 && (((uintptr_t)jb.out & 15) == 0);
    for (int t = threadIdx.x; t < nrow * cq; t += 256) {
        const int r = t / cq, c0 = (t - r * cq) * 4;
        const int row = row0 + r;
        const int kp = row / jb.RS, rs = row - kp * jb.RS;
        const int64_t k = jb.idxK ? jb.idxK[kp] : kp;
        const float* src = jb.w + (k * jb.RS + rs) * (int64_t)jb.cpitch;
        float* dst = jb.out + (int64_t)row * jb.out_cpitch + c0;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int c = c0 + e;
            v[e] = (c < jb.Cp) ? src[jb.idxC ? jb.idxC[c] : c] : 0.f;
        }
        if (c0 + 3 < jb.Cp && vec) {
            *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (c0 + e < jb.Cp) dst[e] = v[e];
        }
    }
}

// ---- channel scatter (inverse of the activation gather), max-abs criterion, zeroing of flagged groups -----

// out[pix][idx[c']] = x[pix][c'], all other channels of out zero.  A workgroup first builds the inverse map
// (source channel or -1 for every output channel) in LDS; a thread then produces 8 consecutive output
// channels of one pixel from up to eight 2-byte reads of that pixel's (contiguous, cached) source row.
constexpr int kScatterMaxC = 8192;
__global__ __launch_bounds__(256) void k_scatter_nhwc(const uint16_t* __restrict__ x, int64_t pixels, int Cp, int x_cpitch,
                                                      const int* __restrict__ idx, int C, uint16_t* __restrict__ out,
                                                      int out_cpitch, int vec_ok) {
    __shared__ short inv[kScatterMaxC];
    for (int c = threadIdx.x; c < C; c += 256) inv[c] = -1;
    __syncthreads();
    for (int b = threadIdx.x; b < Cp; b += 256) inv[idx[b]] = (short)b;
    __syncthreads();
    const int cv = (C + 7) >> 3;
    const int64_t work = pixels * cv;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < work; t += (int64_t)gridDim.x * 256) {
        const int64_t pix = t / cv;
        const int c0 = (int)(t - pix * cv) * 8;
        const uint16_t* src = x + pix * (int64_t)x_cpitch;
        uint16_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int c = c0 + e;
            const int b = c < C ? inv[c] : -1;
            v[e] = b >= 0 ? src[b] : (uint16_t)0;
        }
        uint16_t* dst = out + pix * (int64_t)out_cpitch + c0;
        if (vec_ok && c0 + 7 < C) {
            uint4 o;
            o.x = v[0] | ((uint32_t)v[1] << 16);
            o.y = v[2] | ((uint32_t)v[3] << 16);
            o.z = v[4] | ((uint32_t)v[5] << 16);
            o.w = v[6] | ((uint32_t)v[7] << 16);
            *reinterpret_cast<uint4*>(dst) = o;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (c0 + e < C) dst[e] = v[e];
        }
    }
}

// Largest |w| per filter and per input channel.  |w| >= 0, so the bit patterns order like the values and the
// maxima can be combined with integer atomic max: exact and independent of the order of arrival.
__global__ void k_fill_u32(uint32_t* __restrict__ p, int n, uint32_t v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
constexpr int kMaxAbsMaxC = 2048;  // 256 threads x 8 columns each
__global__ __launch_bounds__(256) void k_group_maxabs(const float* __restrict__ w, int K, int RS, int C, int cpitch,
                                                      uint32_t* __restrict__ out_max, uint32_t* __restrict__ in_max,
                                                      int rows_per_block) {
    // a workgroup owns rows_per_block consecutive (k, rs) rows; thread t keeps columns t, t+256, ... in registers
    const int64_t rows = (int64_t)K * RS;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = min(rows, r0 + rows_per_block);
    uint32_t cm[kMaxAbsMaxC / 256];
#pragma unroll
    for (int j = 0; j < kMaxAbsMaxC / 256; ++j) cm[j] = 0u;
    for (int64_t r = r0; r < r1; ++r) {
        uint32_t rm = 0u;
#pragma unroll
        for (int j = 0; j < kMaxAbsMaxC / 256; ++j) {
            const int c = threadIdx.x + j * 256;
            if (c < C) {
                const uint32_t a = __float_as_uint(fabsf(w[r * cpitch + c]));
                cm[j] = max(cm[j], a);
                rm = max(rm, a);
            }
        }
        for (int off = 32; off > 0; off >>= 1) rm = max(rm, (uint32_t)__shfl_xor((int)rm, off));
        if ((threadIdx.x & 63) == 0) atomicMax(&out_max[r / RS], rm);
    }
#pragma unroll
    for (int j = 0; j < kMaxAbsMaxC / 256; ++j) {
        const int c = threadIdx.x + j * 256;
        if (c < C) atomicMax(&in_max[c], cm[j]);
    }
}

// w[k][rs][c] = 0 where zero_out[k] or zero_in[c] (either mask may be null).
__global__ void k_apply_zero(float* __restrict__ w, int64_t rows, int RS, int C, int cpitch,
                             const uint8_t* __restrict__ zero_out, const uint8_t* __restrict__ zero_in) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= rows * C) return;
    const int64_t r = t / C;
    const int c = (int)(t - r * C);
    const bool z = (zero_out && zero_out[r / RS]) || (zero_in && zero_in[c]);
    if (z) w[r * cpitch + c] = 0.f;
}

}  // namespace pt

using namespace pt;

extern "C" int32_t pt_zero_groups(const float* norms, int32_t n, float thr, uint8_t* zero, void* stream) {
    if (n < 0) return PT_ERR_SHAPE;
    if (n == 0) return PT_OK;
    if (!norms || !zero) return PT_ERR_NULL;
    hipLaunchKernelGGL(k_zero_groups, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, norms, n, thr, zero);
    return launch_status();
}

extern "C" int32_t pt_reconcile_edge(const uint8_t* const* producer_zero, int32_t n_prod,
                                     const uint8_t* const* consumer_zero, int32_t n_cons, int32_t n, uint8_t* keep,
                                     void* stream) {
    if (n < 0 || n_prod < 0 || n_cons < 0 || n_prod + n_cons < 1) return PT_ERR_SHAPE;
    if (n_prod + n_cons > kMaxEdgeMembers) return PT_ERR_UNSUPPORTED;
    if ((n_prod > 0 && !producer_zero) || (n_cons > 0 && !consumer_zero)) return PT_ERR_NULL;
    EdgeMasks e;
    e.count = 0;
    for (int a = 0; a < n_prod; ++a) {
        if (!producer_zero[a]) return PT_ERR_NULL;
        e.m[e.count++] = producer_zero[a];
    }
    for (int a = 0; a < n_cons; ++a) {
        if (!consumer_zero[a]) return PT_ERR_NULL;
        e.m[e.count++] = consumer_zero[a];
    }
    for (int a = e.count; a < kMaxEdgeMembers; ++a) e.m[a] = nullptr;
    if (n == 0) return PT_OK;
    if (!keep) return PT_ERR_NULL;
    hipLaunchKernelGGL(k_reconcile_edge, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, e, n, keep);
    return launch_status();
}

extern "C" int32_t pt_compact_plan(const uint8_t* keep, int32_t n, int32_t* idx, int32_t* n_keep_dev, void* stream) {
    if (n < 0) return PT_ERR_SHAPE;
    if (!n_keep_dev || (n > 0 && (!keep || !idx))) return PT_ERR_NULL;
    hipLaunchKernelGGL(k_compact_plan, dim3(1), dim3(1024), 0, (hipStream_t)stream, keep, n, idx, n_keep_dev);
    return launch_status();
}

extern "C" int32_t pt_compact_weights(const float* w, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch,
                                      const int32_t* idxK, int32_t Kp, const int32_t* idxC, int32_t Cp, float* w_out,
                                      int32_t out_cpitch, void* stream) {
    if (!w || !w_out) return PT_ERR_NULL;
    if (K <= 0 || RS <= 0 || C <= 0 || Kp <= 0 || Cp <= 0 || w_cpitch < C || out_cpitch < Cp) return PT_ERR_SHAPE;
    if ((!idxK && Kp != K) || (!idxC && Cp != C) || Kp > K || Cp > C) return PT_ERR_SHAPE;
    const int64_t out_rows = (int64_t)Kp * RS;
    const int64_t work = out_rows * ((Cp + 3) / 4);
    const int64_t nblk = ceil_div(work, 256);
    if (nblk > 0x7fffffff) return PT_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_compact_weights, dim3((unsigned)nblk), dim3(256), 0, (hipStream_t)stream, w, RS, w_cpitch, idxK,
                       idxC, Cp, out_cpitch, out_rows, w_out);
    return launch_status();
}

extern "C" int32_t pt_compact_vector(const void* v, int32_t elem_bytes, const int32_t* idx, int32_t n_keep, void* out,
                                     void* stream) {
    if (n_keep < 0) return PT_ERR_SHAPE;
    if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8) return PT_ERR_UNSUPPORTED;
    if (n_keep == 0) return PT_OK;
    if (!v || !idx || !out) return PT_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    const dim3 g((n_keep + 255) / 256), b(256);
    switch (elem_bytes) {
        case 1: hipLaunchKernelGGL(k_compact_vector<uint8_t>, g, b, 0, st, (const uint8_t*)v, idx, n_keep, (uint8_t*)out); break;
        case 2: hipLaunchKernelGGL(k_compact_vector<uint16_t>, g, b, 0, st, (const uint16_t*)v, idx, n_keep, (uint16_t*)out); break;
        case 4: hipLaunchKernelGGL(k_compact_vector<uint32_t>, g, b, 0, st, (const uint32_t*)v, idx, n_keep, (uint32_t*)out); break;
        default: hipLaunchKernelGGL(k_compact_vector<uint64_t>, g, b, 0, st, (const uint64_t*)v, idx, n_keep, (uint64_t*)out); break;
    }
    return launch_status();
}

// Host side of the activation gathers: tensors that qualify for the streaming kernel are collected into job
// tables (one launch per kMaxGatherJobs tensors); the others take the element-wise kernel one by one.
static int32_t check_gather(const uint16_t* x, int64_t pixels, int32_t C, int32_t x_cpitch, const int32_t* idx, int32_t Cp,
                            uint16_t* out, int32_t out_cpitch) {
    if (pixels < 0 || C <= 0 || Cp <= 0 || Cp > C || x_cpitch < C || out_cpitch < Cp) return PT_ERR_SHAPE;
    if (pixels > 0 && (!x || !idx || !out)) return PT_ERR_NULL;
    return PT_OK;
}
static bool gather_streams(const uint16_t* x, int32_t x_cpitch, int32_t Cp, const uint16_t* out, int32_t out_cpitch) {
    return (x_cpitch % 8 == 0) && (out_cpitch % 8 == 0) && (((uintptr_t)x & 15) == 0) && (((uintptr_t)out & 15) == 0) &&
           (Cp + 7) / 8 <= kGatherThreads && (size_t)x_cpitch * 2 <= (size_t)kGatherChunk;
}
static int32_t launch_gather_jobs(GatherJobs& t, hipStream_t st) {
    if (t.n == 0) return PT_OK;
    static LdsOptIn opt_in;  // 64 KiB of dynamic LDS
    if (hipError_t e = opt_in.ensure(reinterpret_cast<const void*>(k_compact_nhwc_lds), 2 * kGatherChunk, 0); e != hipSuccess) {
        set_hip_error(e);
        return PT_ERR_LAUNCH;
    }
    const unsigned grid = (unsigned)(t.total_chunks < 512 ? t.total_chunks : 512);  // two resident workgroups per CU
    hipLaunchKernelGGL(k_compact_nhwc_lds, dim3(grid), dim3(kGatherThreads), 2 * kGatherChunk, st, t);
    t.n = 0;
    t.total_chunks = 0;
    return launch_status();
}
static int32_t add_gather_job(GatherJobs& t, const uint16_t* x, int64_t pixels, int32_t x_cpitch, const int32_t* idx,
                              int32_t Cp, uint16_t* out, int32_t out_cpitch, hipStream_t st) {
    // whole pixel rows per LDS buffer, a multiple of the pixels gathered per pass
    const int nvec = (Cp + 7) / 8, ppb = kGatherThreads / nvec;
    int ppc = (int)(kGatherChunk / ((size_t)x_cpitch * 2));
    if (ppc > ppb) ppc = ppc / ppb * ppb;
    const int64_t nchunks = ceil_div(pixels, ppc);
    if (nchunks > 0x3fffffff) return PT_ERR_UNSUPPORTED;
    if (t.n == kMaxGatherJobs || (int64_t)t.total_chunks + nchunks > 0x3fffffff) {
        const int32_t rc = launch_gather_jobs(t, st);
        if (rc != PT_OK) return rc;
    }
    t.j[t.n++] = GatherJob{x, idx, out, pixels, x_cpitch, Cp, out_cpitch, ppc, t.total_chunks, 0};
    t.total_chunks += (int)nchunks;
    return PT_OK;
}
static int32_t gather_elementwise(const uint16_t* x, int64_t pixels, int32_t x_cpitch, const int32_t* idx, int32_t Cp,
                                  uint16_t* out, int32_t out_cpitch, hipStream_t st) {
    const int64_t work = pixels * ((Cp + 7) / 8);
    const int64_t nblk = ceil_div(work, 256);
    if (nblk > 0x7fffffff) return PT_ERR_UNSUPPORTED;
    const int vec_ok = (out_cpitch % 8 == 0) && (((uintptr_t)out & 15) == 0);
    hipLaunchKernelGGL(k_compact_nhwc, dim3((unsigned)nblk), dim3(256), 0, st, x, pixels, x_cpitch, idx, Cp, out,
                       out_cpitch, vec_ok);
    return launch_status();
}

extern "C" int32_t pt_compact_nhwc(const uint16_t* x, int64_t pixels, int32_t C, int32_t x_cpitch, const int32_t* idx,
                                   int32_t Cp, uint16_t* out, int32_t out_cpitch, void* stream) {
    const int32_t rc = check_gather(x, pixels, C, x_cpitch, idx, Cp, out, out_cpitch);
    if (rc != PT_OK) return rc;
    if (pixels == 0) return PT_OK;
    hipStream_t st = (hipStream_t)stream;
    if (!gather_streams(x, x_cpitch, Cp, out, out_cpitch)) return gather_elementwise(x, pixels, x_cpitch, idx, Cp, out, out_cpitch, st);
    GatherJobs t;
    t.n = 0;
    t.total_chunks = 0;
    const int32_t r2 = add_gather_job(t, x, pixels, x_cpitch, idx, Cp, out, out_cpitch, st);
    if (r2 != PT_OK) return r2;
    return launch_gather_jobs(t, st);
}

extern "C" int32_t pt_compact_nhwc_batched(const pt_gather_nhwc* jobs, int32_t n_jobs, void* stream) {
    if (n_jobs < 0) return PT_ERR_SHAPE;
    if (n_jobs == 0) return PT_OK;
    if (!jobs) return PT_ERR_NULL;
    for (int i = 0; i < n_jobs; ++i) {
        const pt_gather_nhwc& j = jobs[i];
        const int32_t rc = check_gather(j.x, j.pixels, j.C, j.x_cpitch, j.idx, j.Cp, j.out, j.out_cpitch);
        if (rc != PT_OK) return rc;
    }
    hipStream_t st = (hipStream_t)stream;
    GatherJobs t;
    t.n = 0;
    t.total_chunks = 0;
    for (int i = 0; i < n_jobs; ++i) {
        const pt_gather_nhwc& j = jobs[i];
        if (j.pixels == 0) continue;
        int32_t rc;
        if (gather_streams(j.x, j.x_cpitch, j.Cp, j.out, j.out_cpitch))
            rc = add_gather_job(t, j.x, j.pixels, j.x_cpitch, j.idx, j.Cp, j.out, j.out_cpitch, st);
        else
            rc = gather_elementwise(j.x, j.pixels, j.x_cpitch, j.idx, j.Cp, j.out, j.out_cpitch, st);
        if (rc != PT_OK) return rc;
    }
    return launch_gather_jobs(t, st);
}

// ---- multi-job entry points ------------------------------------------------------------------------
extern "C" int32_t pt_zero_groups_batched(const pt_norm_mask* jobs, int32_t n_jobs, float thr, void* stream) {
    if (n_jobs < 0) return PT_ERR_SHAPE;
    if (n_jobs == 0) return PT_OK;
    if (!jobs) return PT_ERR_NULL;
    for (int i = 0; i < n_jobs; ++i) {
        if (jobs[i].n < 0) return PT_ERR_SHAPE;
        if (jobs[i].n > 0 && (!jobs[i].norms || !jobs[i].zero)) return PT_ERR_NULL;
    }
    MaskJobs t;
    t.n = 0;
    int blocks = 0;
    auto flush = [&]() -> int32_t {
        if (t.n == 0) return PT_OK;
        hipLaunchKernelGGL(k_zero_groups_multi, dim3(blocks), dim3(256), 0, (hipStream_t)stream, t, thr);
        t.n = 0;
        blocks = 0;
        return launch_status();
    };
    for (int i = 0; i < n_jobs; ++i) {
        if (jobs[i].n == 0) continue;
        t.j[t.n++] = MaskJob{jobs[i].norms, jobs[i].zero, jobs[i].n, blocks};
        blocks += (jobs[i].n + 255) / 256;
        if (t.n == kMaxMaskJobs) {
            const int32_t rc = flush();
            if (rc != PT_OK) return rc;
        }
    }
    return flush();
}

extern "C" int32_t pt_reconcile_plan_batched(const pt_edge_plan* edges, int32_t n_edges, void* stream) {
    if (n_edges < 0) return PT_ERR_SHAPE;
    if (n_edges == 0) return PT_OK;
    if (!edges) return PT_ERR_NULL;
    for (int i = 0; i < n_edges; ++i) {
        const pt_edge_plan& e = edges[i];
        if (e.n < 0 || e.n_prod < 0 || e.n_cons < 0 || e.n_prod + e.n_cons < 1) return PT_ERR_SHAPE;
        if (e.n_prod + e.n_cons > kMaxEdgeMembers) return PT_ERR_UNSUPPORTED;
        if ((e.n_prod > 0 && !e.producer_zero) || (e.n_cons > 0 && !e.consumer_zero) || !e.n_keep_dev) return PT_ERR_NULL;
        if (e.n > 0 && (!e.keep || !e.idx)) return PT_ERR_NULL;
        for (int a = 0; a < e.n_prod; ++a)
            if (!e.producer_zero[a]) return PT_ERR_NULL;
        for (int a = 0; a < e.n_cons; ++a)
            if (!e.consumer_zero[a]) return PT_ERR_NULL;
    }
    PlanJobs t;
    int ne = 0, nm = 0;
    auto flush = [&]() -> int32_t {
        if (ne == 0) return PT_OK;
        for (int a = nm; a < kMaxPlanMembers; ++a) t.m[a] = nullptr;
        hipLaunchKernelGGL(k_reconcile_plan_multi, dim3(ne), dim3(1024), 0, (hipStream_t)stream, t);
        ne = nm = 0;
        return launch_status();
    };
    for (int i = 0; i < n_edges; ++i) {
        const pt_edge_plan& e = edges[i];
        const int mc = e.n_prod + e.n_cons;
        if (ne == kMaxPlanEdges || nm + mc > kMaxPlanMembers) {
            const int32_t rc = flush();
            if (rc != PT_OK) return rc;
        }
        t.e[ne++] = PlanEdge{e.keep, e.idx, e.n_keep_dev, e.n, nm, mc};
        for (int a = 0; a < e.n_prod; ++a) t.m[nm++] = e.producer_zero[a];
        for (int a = 0; a < e.n_cons; ++a) t.m[nm++] = e.consumer_zero[a];
    }
    return flush();
}

extern "C" int32_t pt_compact_vector_batched(const pt_gather_vector* jobs, int32_t n_jobs, void* stream) {
    if (n_jobs < 0) return PT_ERR_SHAPE;
    if (n_jobs == 0) return PT_OK;
    if (!jobs) return PT_ERR_NULL;
    for (int i = 0; i < n_jobs; ++i) {
        const pt_gather_vector& j = jobs[i];
        if (j.n_keep < 0) return PT_ERR_SHAPE;
        if (j.elem_bytes != 1 && j.elem_bytes != 2 && j.elem_bytes != 4 && j.elem_bytes != 8) return PT_ERR_UNSUPPORTED;
        if (j.n_keep > 0 && (!j.v || !j.idx || !j.out)) return PT_ERR_NULL;
    }
    VecJobs t;
    t.n = 0;
    int blocks = 0;
    auto flush = [&]() -> int32_t {
        if (t.n == 0) return PT_OK;
        hipLaunchKernelGGL(k_compact_vector_multi, dim3(blocks), dim3(256), 0, (hipStream_t)stream, t);
        t.n = 0;
        blocks = 0;
        return launch_status();
    };
    for (int i = 0; i < n_jobs; ++i) {
        const pt_gather_vector& j = jobs[i];
        if (j.n_keep == 0) continue;
        t.j[t.n++] = VecJob{j.v, j.idx, j.out, j.n_keep, j.elem_bytes, blocks, 0};
        blocks += (j.n_keep + 255) / 256;
        if (t.n == kMaxVecJobs) {
            const int32_t rc = flush();
            if (rc != PT_OK) return rc;
        }
    }
    return flush();
}

extern "C" int32_t pt_compact_weights_batched(const pt_gather_weights* jobs, int32_t n_jobs, void* stream) {
    if (n_jobs < 0) return PT_ERR_SHAPE;
    if (n_jobs == 0) return PT_OK;
    if (!jobs) return PT_ERR_NULL;
    for (int i = 0; i < n_jobs; ++i) {
        const pt_gather_weights& j = jobs[i];
        if (!j.w || !j.w_out) return PT_ERR_NULL;
        if (j.K <= 0 || j.RS <= 0 || j.C <= 0 || j.Kp <= 0 || j.Cp <= 0 || j.w_cpitch < j.C || j.out_cpitch < j.Cp)
            return PT_ERR_SHAPE;
        if ((!j.idxK && j.Kp != j.K) || (!j.idxC && j.Cp != j.C) || j.Kp > j.K || j.Cp > j.C) return PT_ERR_SHAPE;
        if ((int64_t)j.Kp * j.RS > 0x7fffffff) return PT_ERR_UNSUPPORTED;
    }
    WJobs t;
    t.n = 0;
    int64_t blocks = 0;
    auto flush = [&]() -> int32_t {
        if (t.n == 0) return PT_OK;
        hipLaunchKernelGGL(k_compact_weights_multi, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, t);
        t.n = 0;
        blocks = 0;
        return launch_status();
    };
    for (int i = 0; i < n_jobs; ++i) {
        const pt_gather_weights& j = jobs[i];
        const int out_rows = j.Kp * j.RS;
        // about 4096 output elements per workgroup
        int rpb = 4096 / (((j.Cp + 3) / 4) * 4);
        if (rpb < 1) rpb = 1;
        const int64_t nb = ceil_div(out_rows, rpb);
        if (blocks + nb > 0x3fffffff) {
            const int32_t rc = flush();
            if (rc != PT_OK) return rc;
        }
        t.j[t.n++] = WJob{j.w, j.idxK, j.idxC, j.w_out, j.RS, j.w_cpitch, j.Cp, j.out_cpitch, out_rows, (int)blocks, rpb, 0};
        blocks += nb;
        if (t.n == kMaxWJobs) {
            const int32_t rc = flush();
            if (rc != PT_OK) return rc;
        }
    }
    return flush();
}

// ---- channel scatter, max-abs criterion, zeroing of flagged groups -------------------------------------
extern "C" int32_t pt_scatter_nhwc(const uint16_t* x, int64_t pixels, int32_t Cp, int32_t x_cpitch, const int32_t* idx,
                                   int32_t C, uint16_t* out, int32_t out_cpitch, void* stream) {
    if (pixels < 0 || C <= 0 || Cp <= 0 || Cp > C || x_cpitch < Cp || out_cpitch < C) return PT_ERR_SHAPE;
    if (C > kScatterMaxC) return PT_ERR_UNSUPPORTED;
    if (pixels == 0) return PT_OK;
    if (!x || !idx || !out) return PT_ERR_NULL;
    const int64_t work = pixels * ((C + 7) / 8);
    int64_t nblk = ceil_div(work, 256);
    if (nblk > 256 * 16) nblk = 256 * 16;  // grid-stride: the inverse map is built once per workgroup
    const int vec_ok = (out_cpitch % 8 == 0) && (((uintptr_t)out & 15) == 0);
    hipLaunchKernelGGL(k_scatter_nhwc, dim3((unsigned)nblk), dim3(256), 0, (hipStream_t)stream, x, pixels, Cp, x_cpitch, idx,
                       C, out, out_cpitch, vec_ok);
    return launch_status();
}

extern "C" int32_t pt_group_maxabs(const float* w, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch, float* out_max,
                                   float* in_max, void* stream) {
    if (K <= 0 || RS <= 0 || C <= 0 || w_cpitch < C) return PT_ERR_SHAPE;
    if (C > kMaxAbsMaxC) return PT_ERR_UNSUPPORTED;
    if (!w || !out_max || !in_max) return PT_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)ceil_div(K, 256)), dim3(256), 0, st, (uint32_t*)out_max, K, 0u);
    int32_t rc = launch_status();
    if (rc != PT_OK) return rc;
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)ceil_div(C, 256)), dim3(256), 0, st, (uint32_t*)in_max, C, 0u);
    rc = launch_status();
    if (rc != PT_OK) return rc;
    const int64_t rows = (int64_t)K * RS;
    int rpb = (int)(16384 / C);  // about 16K elements per workgroup
    if (rpb < 1) rpb = 1;
    if (rpb > 256) rpb = 256;
    const int64_t nblk = ceil_div(rows, rpb);
    if (nblk > 0x7fffffff) return PT_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_group_maxabs, dim3((unsigned)nblk), dim3(256), 0, st, w, K, RS, C, w_cpitch, (uint32_t*)out_max,
                       (uint32_t*)in_max, rpb);
    return launch_status();
}

extern "C" int32_t pt_apply_zero(float* w, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch, const uint8_t* zero_out,
                                 const uint8_t* zero_in, void* stream) {
    if (K <= 0 || RS <= 0 || C <= 0 || w_cpitch < C) return PT_ERR_SHAPE;
    if (!w) return PT_ERR_NULL;
    if (!zero_out && !zero_in) return PT_OK;
    const int64_t rows = (int64_t)K * RS;
    const int64_t nblk = ceil_div(rows * C, 256);
    if (nblk > 0x7fffffff) return PT_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_apply_zero, dim3((unsigned)nblk), dim3(256), 0, (hipStream_t)stream, w, rows, RS, C, w_cpitch,
                       zero_out, zero_in);
    return launch_status();
}
