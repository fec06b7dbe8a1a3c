// Device kernels and launch templates of the implicit-GEMM convolutions (gfx950).
// See conv.hip for the map from the three convolution calls onto these kernels.
#pragma once

#include <type_traits>

#include "common.h"

namespace pt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Raw 8 x bf16 load from base + off (elements).  VEC: one 16-byte load (off*2 is 16-byte aligned and all
// 16 bytes are readable).  Otherwise eight 2-byte loads, where element e >= nvalid re-reads element 0 so
// that nothing beyond the row's logical extent is touched.  No branches: callers clamp `off` to a
// readable location for rows that are out of range and zero the result with mask8().
template <bool VEC>
__device__ __forceinline__ uint4 ldg8(const uint16_t* __restrict__ base, uint32_t off, int nvalid) {
    if constexpr (VEC) {
        return *reinterpret_cast<const uint4*>(base + off);
    } else {
        uint32_t d[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t lo = base[off + (2 * i < nvalid ? 2 * i : 0)];
            const uint32_t hi = base[off + (2 * i + 1 < nvalid ? 2 * i + 1 : 0)];
            d[i] = lo | (hi << 16);
        }
        return make_uint4(d[0], d[1], d[2], d[3]);
    }
}

// Per-dword masks that keep elements [0, nvalid) of an 8 x bf16 vector.
struct Mask8 {
    uint32_t m[4];
};
__device__ __forceinline__ Mask8 make_mask8(int nvalid) {
    Mask8 k;
#pragma unroll
    for (int i = 0; i < 4; ++i) k.m[i] = nvalid >= 2 * i + 2 ? 0xffffffffu : (nvalid == 2 * i + 1 ? 0xffffu : 0u);
    return k;
}
__device__ __forceinline__ uint4 mask8(uint4 v, bool ok, const Mask8& k) {
    v.x = ok ? (v.x & k.m[0]) : 0u;
    v.y = ok ? (v.y & k.m[1]) : 0u;
    v.z = ok ? (v.z & k.m[2]) : 0u;
    v.w = ok ? (v.w & k.m[3]) : 0u;
    return v;
}

// LDS reads issued as inline assembly are ordered only by explicit waits: the compiler neither moves them nor
// adds waits of its own.  The result registers must not be touched before lds_wait() has been applied to them.
// Waits until at most N of this wave's LDS reads are outstanding (they return in order) and makes `first`
// depend on the wait; lds_tie() extends the dependence to further registers.
template <int N, typename V>
__device__ __forceinline__ void lds_wait(V& first) {
    static_assert(N >= 0 && N < 16, "lgkmcnt range");
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(first) : "n"(N));
}
template <typename V>
__device__ __forceinline__ void lds_tie(V& v) {
    asm volatile("" : "+v"(v));
}
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// XCD-aware block remap: hardware deals consecutive workgroup ids round-robin to the 8 XCDs; give
// each XCD a contiguous range of logical tiles so tiles that share operands share an L2.
__device__ __forceinline__ int xcd_remap(int bid, int nb) {
    const int xcd = bid & 7, q = bid >> 3;
    const int per = nb >> 3, rem = nb & 7;
    return xcd * per + min(xcd, rem) + q;
}

// floor(m / d) through a host-made magic number (exact for m * d < 2^32); d == 1 has magic 0.
struct FastDiv {
    uint32_t d, magic;
};
inline FastDiv make_fastdiv(uint32_t d) { return FastDiv{d, d == 1 ? 0u : make_magic(d)}; }
__device__ __forceinline__ uint32_t fdiv(uint32_t m, FastDiv f) { return f.d == 1 ? m : __umulhi(m, f.magic); }

// ------------------------------------------------------------------------------------------- //
// forward / input-gradient implicit GEMM
// ------------------------------------------------------------------------------------------- //
struct IgemmArgs {
    const uint16_t* A;  // gathered activations (x or dy)
    const uint16_t* B;  // weights, [Nout][b_taps][bpitch], reduction channel innermost
    uint16_t* D;        // output activations
    int M;              // output pixels of this launch = images * gH * gW
    FastDiv gW, gH;     // output pixel grid per image (of this launch): width, height
    int srcH, srcW, apitch;
    int h_mul, h_add, w_mul, w_add;  // source coordinate of tap (0,0) for grid point (i,j)
    int tr_step, ts_step;            // source coordinate step per tap index
    int TR, TS;                      // taps of this launch
    int Cred, CredP;                 // reduction channels, and rounded up to 8
    // Folded small-channel mode (direct kernel only): when a pixel holds fewer than 64 padded channels and
    // pixels are dense (pitch == padded channels), the S taps of a filter row are one contiguous run of
    // S*Cfold elements in both operands, so a reduction step covers several taps.  Then TS == 1,
    // Cred == CredP == S*Cfold, TSm == S taps per row in the validity mask, Creal real channels per tap.
    int fold, TSm, Creal;
    FastDiv Cfold;
    int b_tap0, b_tr_stride, b_ts_stride, b_taps;
    int bpitch, Nout;
    int DH, DW, d_hmul, d_hadd, d_wmul, d_wadd, dpitch;  // destination pixel = (i*d_hmul+d_hadd, j*d_wmul+d_wadd)
    int d_linear;                                        // destination pixel index == m
    int nk;                                              // reduction steps of BK
    int tiles_n;
    int d_vec;    // 8-byte stores allowed (pitch % 4 == 0, base 8-byte aligned)
    int d_vec16;  // 16-byte stores allowed (pitch % 8 == 0, base 16-byte aligned)
    // Direct kernel, channel counts that are not multiples of 8: which of the eight 16-byte chunks of a 64-channel block
    // end in undefined padding elements.  Byte b of tail_kv = chunk bits of block b of a folded run; otherwise byte 0
    // describes the last block of a tap (the only one with a tail) and byte 7 is zero.
    uint64_t tail_kv;
    int tail_nvalid;  // defined elements of a tail chunk (1..7), 8 when there is none
    int pad_zero;     // the caller vouches that the padding channels of both operands hold zeros
    // Input gradient of a strided layer whose only stride-parity class with filter taps is (0, 0): every destination
    // pixel lies in the zf_h x zf_w cell anchored at one pixel of that class, and the launch clears the rest of each
    // cell itself (1 x 1 = off).  Direct kernel, 16-byte stores only.
    int zf_h, zf_w;
    // STATS instantiations (forward only): per-channel sums of the stored (bf16-rounded) outputs and of their
    // squares over the tile's valid pixels, one row per pixel tile: stats[(q * tiles_m + tile_m) * Nout + channel],
    // q = 0 sums, q = 1 sums of squares - the layout the normalisation's finish pass reads.
    float* stats;
    int tiles_m;
    // Direct kernel, buffer addressing of the gathered operand: a row's offset plus a_guard is non-negative for
    // every row, a reduction step's offset minus a_smin is non-negative for every step (both in elements; the
    // buffer's base address absorbs the two shifts).  a_all_valid: no tap of any row ever leaves the source image.
    int a_guard, a_smin, a_all_valid;
    // Direct kernel: wave priority outside the reduction loop (inside it is 2).  0 for a launch that runs alone; the
    // input gradient, which is meant to run beside weight gradients of other layers, keeps its set-up and its stores
    // ahead of them too.
    int edge_prio;
    int grid_x;  // direct kernel: workgroups (tiles) of this problem inside a launch that may hold several problems
};

// The direct kernel takes up to four problems per launch, one per blockIdx.y (the stride-parity classes of a strided
// input gradient: disjoint output pixels, the same operands): workgroups past a problem's own tile count leave at once.
constexpr int kIgemmMaxProblems = 4;
struct IgemmArgsN {
    IgemmArgs a[kIgemmMaxProblems];
};

// Fills tail_kv / tail_nvalid (see IgemmArgs) for the direct kernel's 64-channel blocks.
inline void set_tail_tables(IgemmArgs& a) {
    a.tail_kv = 0;
    a.tail_nvalid = 8;
    const int creal = a.fold ? a.Creal : a.Cred;
    if ((creal & 7) == 0) return;
    a.tail_nvalid = creal & 7;
    const int tail_chunk = creal >> 3;  // chunk index of the tail inside one run
    if (!a.fold) {
        a.tail_kv = 1ull << (tail_chunk & 7);  // in the last block of the tap
        return;
    }
    const int per = (int)(a.Cfold.d >> 3);  // chunks per run
    const int nblk = (a.CredP + 63) >> 6;   // <= 7
    for (int c = 0; c < nblk * 8; ++c)
        if (c % per == tail_chunk) a.tail_kv |= 1ull << c;
}

// VEC: every operand row is 16-byte aligned (pitches are multiples of 8 elements).
template <int BM, int BN, int BK, int WGM, int WGN, int STAGES, int MINB, bool VEC>
__global__ __launch_bounds__(64 * WGM * WGN, MINB) void k_igemm(const IgemmArgs a) {
    constexpr int NT = 64 * WGM * WGN;
    constexpr int LDK = BK + 8;  // LDS row pitch in elements (16-byte pad: conflict-free 16-byte reads)
    constexpr int KV = BK / 8;
    constexpr int RPP = NT / KV;
    constexpr int AP = BM / RPP, BP = BN / RPP;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int STAGE_ELEMS = (BM + BN) * LDK;
    static_assert(AP >= 1 && BP >= 1 && TM >= 1 && TN >= 1 && BM % RPP == 0 && BN % RPP == 0, "tile config");
    static_assert(STAGES == 1 || STAGES == 2, "stages");
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int n0 = (tile % a.tiles_n) * BN;
    const int m0 = (tile / a.tiles_n) * BM;

    // ---- loader state -------------------------------------------------------------------------
    const int kv = tid % KV, lrow = tid / KV;
    int c0 = kv * 8, tr = 0, ts = 0;
    while (c0 >= a.CredP) {
        c0 -= a.CredP;
        if (++ts == a.TS) { ts = 0; ++tr; }
    }
    int a_hw[AP];    // (h0 << 16) | (w0 & 0xffff): source coordinate of tap (0,0)
    int a_poff[AP];  // linear source pixel of tap (0,0)
#pragma unroll
    for (int i = 0; i < AP; ++i) {
        const int m = m0 + lrow + i * RPP;
        int h0 = -30000, w0 = 0, poff = 0;
        if (m < a.M) {
            const uint32_t row = fdiv((uint32_t)m, a.gW), gj = m - row * a.gW.d;
            const uint32_t n = fdiv(row, a.gH), gi = row - n * a.gH.d;
            h0 = (int)gi * a.h_mul + a.h_add;
            w0 = (int)gj * a.w_mul + a.w_add;
            poff = ((int)n * a.srcH + h0) * a.srcW + w0;
        }
        a_hw[i] = (h0 << 16) | (w0 & 0xffff);
        a_poff[i] = poff;
    }
    const uint32_t b_rowlen = (uint32_t)a.b_taps * a.bpitch;

    uint4 ra[AP], rb[BP];
    bool oka[AP], okb[BP];
    Mask8 kmask;
    // issue the global loads of the next reduction step (raw, unmasked)
    auto gload = [&]() {
        const bool kok = tr < a.TR;
        const int nvalid = kok ? a.Cred - c0 : 0;
        kmask = make_mask8(nvalid);
        const int dh = tr * a.tr_step, dw = ts * a.ts_step;
        const int dpix = dh * a.srcW + dw;
#pragma unroll
        for (int i = 0; i < AP; ++i) {
            const int ih = (a_hw[i] >> 16) + dh, iw = (int)(short)(a_hw[i] & 0xffff) + dw;
            oka[i] = kok && (unsigned)ih < (unsigned)a.srcH && (unsigned)iw < (unsigned)a.srcW;
            const uint32_t off = (uint32_t)(a_poff[i] + dpix) * (uint32_t)a.apitch + (uint32_t)c0;
            ra[i] = ldg8<VEC>(a.A, oka[i] ? off : 0u, nvalid);
        }
        const uint32_t tapoff = (uint32_t)(a.b_tap0 + tr * a.b_tr_stride + ts * a.b_ts_stride) * (uint32_t)a.bpitch + c0;
#pragma unroll
        for (int j = 0; j < BP; ++j) {
            const int nrow = n0 + lrow + j * RPP;
            okb[j] = kok && nrow < a.Nout;
            rb[j] = ldg8<VEC>(a.B, okb[j] ? (uint32_t)nrow * b_rowlen + tapoff : 0u, nvalid);
        }
        c0 += BK;
        while (c0 >= a.CredP && tr < a.TR) {
            c0 -= a.CredP;
            if (++ts == a.TS) { ts = 0; ++tr; }
        }
    };
    auto sstore = [&](int buf) {
        uint16_t* sA = smem + buf * STAGE_ELEMS;
        uint16_t* sB = sA + BM * LDK;
#pragma unroll
        for (int i = 0; i < AP; ++i)
            *reinterpret_cast<uint4*>(&sA[(lrow + i * RPP) * LDK + kv * 8]) = mask8(ra[i], oka[i], kmask);
#pragma unroll
        for (int j = 0; j < BP; ++j)
            *reinterpret_cast<uint4*>(&sB[(lrow + j * RPP) * LDK + kv * 8]) = mask8(rb[j], okb[j], kmask);
    };

    // ---- MFMA state ---------------------------------------------------------------------------
    const int wm = wave % WGM, wn = wave / WGM;
    const int l32 = lane & 31, lk = (lane >> 5) * 8;
    f32x16 acc[TN][TM];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tn][tm][v] = 0.f;
    bool n_live[TN], m_live[TM];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) n_live[tn] = n0 + wn * WTN + tn * 32 < a.Nout;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) m_live[tm] = m0 + wm * WTM + tm * 32 < a.M;

    bool all_live = true;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) all_live = all_live && n_live[tn];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) all_live = all_live && m_live[tm];

    // CHECK = false: every 32x32 block of this wave is inside the output (no per-block tests)
    auto compute = [&](int buf, auto check_tag) {
        constexpr bool CHECK = decltype(check_tag)::value;
        const uint16_t* sA = smem + buf * STAGE_ELEMS;
        const uint16_t* sB = sA + BM * LDK;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fw[TN], fp[TM];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                fw[tn] = *reinterpret_cast<const bf16x8*>(&sB[(wn * WTN + tn * 32 + l32) * LDK + ks * 16 + lk]);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                fp[tm] = *reinterpret_cast<const bf16x8*>(&sA[(wm * WTM + tm * 32 + l32) * LDK + ks * 16 + lk]);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    if (!CHECK || (n_live[tn] && m_live[tm]))
                        acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[tn], fp[tm], acc[tn][tm], 0, 0, 0);
        }
    };
    // software pipeline over the reduction steps; the tile-edge test is hoisted out of the loop
    auto main_loop = [&](auto check_tag) {
        if constexpr (STAGES == 2) {
            for (int kt = 0; kt < a.nk; ++kt) {
                const int buf = kt & 1;
                if (kt + 1 < a.nk) gload();
                compute(buf, check_tag);
                if (kt + 1 < a.nk) sstore(buf ^ 1);
                __syncthreads();
            }
        } else {
            for (int kt = 0; kt < a.nk; ++kt) {
                if (kt + 1 < a.nk) gload();
                compute(0, check_tag);
                __syncthreads();
                if (kt + 1 < a.nk) {
                    sstore(0);
                    __syncthreads();
                }
            }
        }
    };
    gload();
    sstore(0);
    __syncthreads();
    if (all_live) main_loop(std::false_type{});
    else main_loop(std::true_type{});

    // ---- epilogue: lane holds pixel (column) l32, channels 8g + 4*(lane/32) + {0..3} of each block --
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int m = m0 + wm * WTM + tm * 32 + l32;
        if (m >= a.M) continue;
        int64_t dpix;
        if (a.d_linear) {
            dpix = (int64_t)m * a.dpitch;
        } else {
            const uint32_t row = fdiv((uint32_t)m, a.gW), gj = m - row * a.gW.d;
            const uint32_t n = fdiv(row, a.gH), gi = row - n * a.gH.d;
            dpix = (((int64_t)n * a.DH + (int)gi * a.d_hmul + a.d_hadd) * a.DW + (int)gj * a.d_wmul + a.d_wadd) * a.dpitch;
        }
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int ch = n0 + wn * WTN + tn * 32 + 8 * g + (lane >> 5) * 4;
                if (ch >= a.Nout) continue;
                const float v0 = acc[tn][tm][4 * g + 0], v1 = acc[tn][tm][4 * g + 1];
                const float v2 = acc[tn][tm][4 * g + 2], v3 = acc[tn][tm][4 * g + 3];
                uint16_t* dst = a.D + dpix + ch;
                if (a.d_vec && ch + 3 < a.Nout) {
                    uint2 o;
                    o.x = pack_bf16x2(v0, v1);
                    o.y = pack_bf16x2(v2, v3);
                    *reinterpret_cast<uint2*>(dst) = o;
                } else {
                    dst[0] = f32_to_bf16(v0);
                    if (ch + 1 < a.Nout) dst[1] = f32_to_bf16(v1);
                    if (ch + 2 < a.Nout) dst[2] = f32_to_bf16(v2);
                    if (ch + 3 < a.Nout) dst[3] = f32_to_bf16(v3);
                }
            }
        }
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, int STAGES, int MINB, bool VEC = true>
inline hipError_t launch_igemm_cfg(IgemmArgs& a, hipStream_t st) {
    constexpr int NT = 64 * WGM * WGN;
    constexpr size_t lds = (size_t)STAGES * (BM + BN) * (BK + 8) * 2;
    auto kern = k_igemm<BM, BN, BK, WGM, WGN, STAGES, MINB, VEC>;
    static LdsOptIn opt_in;
    if (hipError_t e = opt_in.ensure(reinterpret_cast<const void*>(kern), lds); e != hipSuccess) return e;
    const int tiles_m = (int)ceil_div(a.M, BM);
    a.tiles_n = (int)ceil_div(a.Nout, BN);
    a.nk = (int)ceil_div((int64_t)a.TR * a.TS * a.CredP, BK);
    hipLaunchKernelGGL(kern, dim3(tiles_m * a.tiles_n), dim3(NT), lds, st, a);
    return hipSuccess;
}

// ------------------------------------------------------------------------------------------- //
// forward / input-gradient implicit GEMM with direct global->LDS loads (vector path)
// ------------------------------------------------------------------------------------------- //
// Same problem mapping as k_igemm, different data movement: 16-byte loads land in LDS without
// passing through registers (buffer_load_dwordx4 ... lds), so several reduction steps can be in flight
// per workgroup at no register cost.  A wave-level load fills 1 KiB of LDS contiguously (lane l ->
// bytes [16l, 16l+16)), i.e. 8 tile rows of BK = 64 elements; rows are unpadded and the eight 16-byte
// chunks of a row are XOR-swizzled with ((row >> 1) & 7) so that the MFMA operand reads (16 consecutive
// rows, same logical chunk) fall into 16 different bank groups.  The swizzle is applied on the global
// side: the lane that owns physical chunk p of a row fetches logical chunk p ^ swz(row).
// Taps outside the image and chunks past the channel count are fetched as zeros (an out-of-range buffer offset, see
// the kernel).  RAGGED = the channel count is not a multiple of 64 (the last block of a run is partly zeros); TAIL = in
// addition some 8-chunk ends in undefined padding elements, which are cleared in LDS before the stage is published.
// The 16-byte zero page below serves the weight-gradient kernel's general gather, which still uses per-lane addresses.
__device__ __attribute__((aligned(16))) uint32_t g_zero16[4] = {0u, 0u, 0u, 0u};

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* glb_void_ptr;

// Workgroup barrier without the memory fence of __syncthreads(): the fence would wait for every
// outstanding global->LDS load, which is exactly what the software pipeline must not do.  Callers
// wait explicitly (vmcnt for landed DMA data, lgkmcnt for their own LDS writes) before calling.
__device__ __forceinline__ void barrier_nofence() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Per-lane choice between two global addresses, kept opaque so that it stays one load instruction.
__device__ __forceinline__ glb_void_ptr pick_ptr(bool ok, const uint16_t* p, const uint16_t* z) {
    uint64_t v = ok ? (uint64_t)(uintptr_t)p : (uint64_t)(uintptr_t)z;
    asm volatile("" : "+v"(v));
    return (glb_void_ptr)(uintptr_t)v;
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    // s_waitcnt immediate: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14 ; only vmcnt constrained
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// TAIL = some run of channels ends inside an 8-chunk whose remaining elements are undefined.
// STATS = also reduce the stored outputs to per-channel sums and sums of squares (see IgemmArgs::stats).
// AV = the caller has established that every tap of every row lies inside the source image (no validity tests).
template <int BM, int BN, int WGM, int WGN, int STAGES, bool RAGGED, bool TAIL = RAGGED, bool STATS = false, bool AV = false>
__global__ __launch_bounds__(64 * WGM * WGN, 1) void k_igemm_dl(const IgemmArgsN problems) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub
    const IgemmArgs a = problems.a[blockIdx.y];  // (a copy: the fields then live in scalar registers as kernel arguments do)
    if (blockIdx.x >= (unsigned)a.grid_x) return;  // the whole workgroup: the launch is as wide as its largest problem
    if (a.edge_prio == 2) __builtin_amdgcn_s_setprio(2);
    else if (a.edge_prio == 1) __builtin_amdgcn_s_setprio(1);
    constexpr int NW = WGM * WGN, BK = 64;
    constexpr int GA = BM / 8, GB = BN / 8;    // 8-row groups = wave-level loads per stage
    constexpr int LA = GA / NW, LB = GB / NW;  // loads per lane per stage
    constexpr int LPT = LA + LB;
    constexpr int STAGE_BYTES = (BM + BN) * 128;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert(NW % 2 == 0 && GA % NW == 0 && GB % NW == 0 && LA >= 1 && LB >= 1 && TM >= 1 && TN >= 1, "tile config");
    static_assert(STAGES >= 2 && (STAGES - 2) * LPT < 64, "stages");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_b[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile = xcd_remap(blockIdx.x, a.grid_x);
    const int n0 = (tile % a.tiles_n) * BN;
    const int m0 = (tile / a.tiles_n) * BM;

    // A reduction step is (filter tap, block of 64 reduction channels): the same for every lane, so the
    // tap offsets and the channel base live in scalar registers.
    const int lrow = lane >> 3;                                      // row inside an 8-row group
    const int kv = (lane & 7) ^ ((((wave & 1) << 2) | (lane >> 4)));  // logical 8-element chunk this lane fetches
    const int kvoff = kv * 8;

    // per-lane row constants: element offset of tap (0,0) + chunk, and a bit per tap: tap inside the image.
    // Rows past the end of the problem are clamped to the last row: their results are never stored.
    uint32_t a_off[LA];
    uint64_t a_mask[LA];  // bit (r * TSm + s): tap (r, s) of this row lies inside the image
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        const int m = min(m0 + (wave + NW * j) * 8 + lrow, a.M - 1);
        const uint32_t row = fdiv((uint32_t)m, a.gW), gj = m - row * a.gW.d;
        const uint32_t n = fdiv(row, a.gH), gi = row - n * a.gH.d;
        const int h0 = (int)gi * a.h_mul + a.h_add, w0 = (int)gj * a.w_mul + a.w_add;
        a_off[j] = (uint32_t)(((int)n * a.srcH + h0) * a.srcW + w0) * (uint32_t)a.apitch + (uint32_t)kvoff;
        // validity is separable: one bit per filter column, replicated for every valid filter row
        uint32_t colbits = 0;
        for (int t = 0; t < a.TSm; ++t) colbits |= ((unsigned)(w0 + t * a.ts_step) < (unsigned)a.srcW ? 1u : 0u) << t;
        uint64_t mask = 0;
        for (int r = 0; r < a.TR; ++r)
            if ((unsigned)(h0 + r * a.tr_step) < (unsigned)a.srcH) mask |= (uint64_t)colbits << (r * a.TSm);
        a_mask[j] = mask;
    }
    const uint32_t b_rowlen = (uint32_t)a.b_taps * a.bpitch;
    uint32_t b_off[LB];
#pragma unroll
    for (int j = 0; j < LB; ++j) {
        const int nrow = min(n0 + (wave + NW * j) * 8 + lrow, a.Nout - 1);
        b_off[j] = (uint32_t)nrow * b_rowlen + (uint32_t)kvoff;
    }
    // Both operands are fetched with buffer loads: the per-lane part of an address (row, 8-element chunk) is a
    // constant byte offset (voffset), the part that changes from step to step (filter tap, channel block) is the same
    // for every lane and travels in a scalar register (soffset), and a lane that must read zeros (tap outside the
    // image, chunk past the channel count) passes an out-of-range voffset, for which the load writes zeros to LDS.
    // The reduction loop is bound by the number of instructions a wave issues, so a step costs no vector arithmetic
    // beyond those validity tests.  The base address of the gathered operand is shifted so that both parts are
    // non-negative (it may point outside the tensor: only valid taps are ever fetched).
    constexpr uint32_t kBufRecords = 0xffffff00u, kBufOut = 0xffffffffu, kBufFlags = 0x00020000u;
    const __amdgpu_buffer_rsrc_t a_srd = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(a.A) + ((int64_t)a.a_smin - a.a_guard), 0, kBufRecords, kBufFlags);
    const __amdgpu_buffer_rsrc_t b_srd = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.B), 0, kBufRecords, kBufFlags);
    uint32_t a_v[LA], b_v[LB];
#pragma unroll
    for (int j = 0; j < LA; ++j) a_v[j] = (a_off[j] + (uint32_t)a.a_guard) * 2u;
#pragma unroll
    for (int j = 0; j < LB; ++j) b_v[j] = b_off[j] * 2u;

    int i_tr = 0, i_ts = 0, i_cb = 0;  // next step to issue (uniform)
    int c_cb = 0;                      // channel base of the next step to compute (uniform)

    auto issue = [&](int stage) {
        uint8_t* sbase = smem_b + stage * STAGE_BYTES;
        const uint32_t sa = (uint32_t)(((i_tr * a.tr_step * a.srcW + i_ts * a.ts_step) * a.apitch + i_cb - a.a_smin) * 2);
        const uint32_t sb = (uint32_t)(((a.b_tap0 + i_tr * a.b_tr_stride + i_ts * a.b_ts_stride) * a.bpitch + i_cb) * 2);
        const bool chunk_ok = !RAGGED || (i_cb + kvoff < a.Cred);
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            uint32_t v = a_v[j];
            if constexpr (!AV) {
                // which tap this lane's chunk belongs to: the step's tap, or in folded mode the tap inside the run
                const int tapbit = i_tr * a.TSm + (a.fold ? (int)fdiv((uint32_t)(i_cb + kvoff), a.Cfold) : i_ts);
                v = (chunk_ok && ((a_mask[j] >> tapbit) & 1u)) ? v : kBufOut;
            } else if constexpr (RAGGED) {
                v = chunk_ok ? v : kBufOut;
            }
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_srd, (lds_void_ptr)(sbase + (wave + NW * j) * 1024), 16, v, sa, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            uint32_t v = b_v[j];
            if constexpr (RAGGED) v = chunk_ok ? v : kBufOut;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(b_srd, (lds_void_ptr)(sbase + BM * 128 + (wave + NW * j) * 1024), 16, v, sb, 0, 0);
        }
        i_cb += BK;
        if (i_cb >= a.CredP) {
            i_cb = 0;
            if (++i_ts == a.TS) { i_ts = 0; ++i_tr; }
        }
    };
    // ---- MFMA state ---------------------------------------------------------------------------
    const int wm = wave % WGM, wn = wave / WGM;
    const int l32 = lane & 31;
    const int swz = (l32 >> 1) & 7;  // all operand rows of this lane are l32 (mod 32)
    const int kc0 = lane >> 5;
    f32x16 acc[TN][TM];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tn][tm][v] = 0.f;
    bool n_live[TN], m_live[TM];
    bool all_live = true;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        n_live[tn] = n0 + wn * WTN + tn * 32 < a.Nout;
        all_live = all_live && n_live[tn];
    }
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        m_live[tm] = m0 + wm * WTM + tm * 32 < a.M;
        all_live = all_live && m_live[tm];
    }

    auto compute = [&](int stage, auto check_tag) {
        constexpr bool CHECK = decltype(check_tag)::value;
        const uint8_t* sA = smem_b + stage * STAGE_BYTES;
        const uint8_t* sB = sA + BM * 128;
        // One stage = BK/16 sub-steps of (fragment reads, MFMAs); all sub-steps always run (chunks past the channel
        // count were fetched as zeros) and the body has no branches: a branch per sub-step costs the
        // compiler's schedule far more than the work it would skip.
        bf16x8 fw[2][TN], fp[2][TM];
        auto read_frags = [&](int ks, int b) {
            const int pc = (((ks * 2 + kc0) ^ swz) << 4);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                fw[b][tn] = *reinterpret_cast<const bf16x8*>(sB + (wn * WTN + tn * 32 + l32) * 128 + pc);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                fp[b][tm] = *reinterpret_cast<const bf16x8*>(sA + (wm * WTM + tm * 32 + l32) * 128 + pc);
        };
        read_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16) read_frags(ks + 1, (ks + 1) & 1);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    if (!CHECK || (n_live[tn] && m_live[tm]))
                        acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[ks & 1][tn], fp[ks & 1][tm], acc[tn][tm],
                                                                              0, 0, 0);
        }
        c_cb += BK;
        if (c_cb >= a.CredP) c_cb = 0;
    };

    // TAIL: a channel count that is not a multiple of 8 leaves undefined elements (memory padding) at the end of the
    // last 8-chunk of every run of channels, in both operands.  The lane that fetched such a chunk overwrites them
    // with zeros in LDS once its loads have landed (writes only: nothing is read back) and before the barrier that
    // publishes the stage.  Which chunks of the current block have a tail comes from a table in the arguments.
    auto clear_tails = [&](int stage) {
        asm volatile("" ::: "memory");  // keep the stores below behind the wait for the landed loads
        const int slot = a.fold ? (c_cb >> 6) : (c_cb + BK > a.Cred ? 0 : 7);
        const uint32_t bits = (uint32_t)(a.tail_kv >> (slot * 8)) & 0xffu;
        if (bits == 0) return;  // wave-uniform
        if ((bits >> kv) & 1u) {
            const int n = a.tail_nvalid;  // uniform, 1..7: bytes [2n, 16) of the chunk are cleared with <= 3 stores
            uint8_t* mine = smem_b + stage * STAGE_BYTES + wave * 1024 + lane * 16;
#pragma unroll
            for (int j = 0; j < LA + LB; ++j) {
                uint8_t* p = mine + (j < LA ? NW * j * 1024 : BM * 128 + NW * (j - LA) * 1024);
                int e = n;
                if (e & 1) {
                    *reinterpret_cast<uint16_t*>(p + 2 * e) = 0;
                    ++e;
                }
                if (e & 2) {
                    *reinterpret_cast<uint32_t*>(p + 2 * e) = 0u;
                    e += 2;
                }
                if (e == 4) *reinterpret_cast<uint64_t*>(p + 8) = 0ull;
            }
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the clears are in LDS before the barrier
    };

    const int nk = a.nk;
    auto main_loop = [&](auto check_tag) {
        for (int kt0 = 0; kt0 < nk; kt0 += STAGES) {
#pragma unroll
            for (int s = 0; s < STAGES; ++s) {
                const int kt = kt0 + s;
                if (kt < nk) {
                    // loads of steps kt+1 .. kt+STAGES-2 may stay in flight; near the end just drain
                    if (kt + STAGES - 2 < nk) wait_vmcnt<(STAGES - 2) * LPT>();
                    else wait_vmcnt<0>();
                    if constexpr (TAIL) clear_tails(s);
                    barrier_nofence();  // stage s complete for every wave; stage (s-1) free again
                    if (kt + STAGES - 1 < nk) issue((s + STAGES - 1) % STAGES);
                    compute(s, check_tag);
                }
            }
        }
    };
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        if (s < nk) issue(s);
    // waves inside the reduction loop go first at the CU's issue arbiter: ahead of a co-resident workgroup's set-up
    // or stores, and ahead of weight-gradient waves sharing the CU from another stream (+0.4 % on the step)
    __builtin_amdgcn_s_setprio(2);
    if (all_live) main_loop(std::false_type{});
    else main_loop(std::true_type{});
    if (a.edge_prio == 0) __builtin_amdgcn_s_setprio(0);
    else if (a.edge_prio == 1) __builtin_amdgcn_s_setprio(1);

    // ---- epilogue: registers -> global.  A lane holds, per 32x32 block, channels 8g + 4*(lane/32) + {0..3}
    // (g = 0..3) of pixel lane%32.  Swapping the upper half-wave of the g-even registers with the lower
    // half-wave of the g-odd ones leaves every lane with two runs of 8 consecutive channels (16 bytes of bf16).
    // Plain launches (16-byte stores, nothing else to write, every chunk a vector) first trade chunks between
    // neighbouring lanes: lane pair (2i, 2i+1) holds chunks (g-pair 0, g-pair 1) of pixels 2i and 2i+1; after the
    // exchange the even lane's pixel is written by both lanes in the first store and the odd lane's in the second,
    // so one store instruction covers 64 contiguous bytes of 16 pixels instead of 32 bytes of 32 pixels (half as
    // many partial-line write requests; a store-only probe of the two patterns differs by 15-25 %).
    const bool pair_store = a.d_vec16 && a.zf_h * a.zf_w == 1 && (a.Nout % 8 == 0 || a.pad_zero);  // uniform
    if (pair_store) {
        const int hi = lane >> 5;
        const bool odd = (l32 & 1) != 0;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int m = m0 + wm * WTM + tm * 32 + l32;
            int64_t dpix;
            if (a.d_linear) {
                dpix = (int64_t)m * a.dpitch;
            } else {
                const uint32_t mm = (uint32_t)min(m, a.M - 1);
                const uint32_t row = fdiv(mm, a.gW), gj = mm - row * a.gW.d;
                const uint32_t n = fdiv(row, a.gH), gi = row - n * a.gH.d;
                const int dh = (int)gi * a.d_hmul + a.d_hadd, dw = (int)gj * a.d_wmul + a.d_wadd;
                dpix = (((int64_t)n * a.DH + dh) * a.DW + dw) * a.dpitch;
            }
            const int64_t dother = ((int64_t)__shfl_xor((int)(dpix >> 32), 1, 64) << 32) |
                                   (uint32_t)__shfl_xor((int)(uint32_t)dpix, 1, 64);
            const int64_t dp0 = odd ? dother : dpix, dp1 = odd ? dpix : dother;  // pixels (m & ~1), (m & ~1) + 1
            const bool ok0 = (m & ~1) < a.M, ok1 = (m | 1) < a.M;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int chb = n0 + wn * WTN + tn * 32;
                if (chb >= a.Nout) continue;  // wave-uniform
                const f32x16& c = acc[tn][tm];
                uint32_t v[2][4];  // this lane's chunk of each register pair: channels chb + 16 gp + 8 hi + {0..7}
#pragma unroll
                for (int gp = 0; gp < 2; ++gp) {
                    const uint32_t p0 = cvt_pk_bf16(c[8 * gp + 0], c[8 * gp + 1]), q0 = cvt_pk_bf16(c[8 * gp + 2], c[8 * gp + 3]);
                    const uint32_t p1 = cvt_pk_bf16(c[8 * gp + 4], c[8 * gp + 5]), q1 = cvt_pk_bf16(c[8 * gp + 6], c[8 * gp + 7]);
                    const auto ps = __builtin_amdgcn_permlane32_swap(p0, p1, false, false);
                    const auto qs = __builtin_amdgcn_permlane32_swap(q0, q1, false, false);
                    v[gp][0] = ps[0]; v[gp][1] = qs[0]; v[gp][2] = ps[1]; v[gp][3] = qs[1];
                }
                uint32_t s0[4], s1[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t give = odd ? v[0][e] : v[1][e];
                    const uint32_t got = (uint32_t)__shfl_xor((int)give, 1, 64);
                    s0[e] = odd ? got : v[0][e];
                    s1[e] = odd ? v[1][e] : got;
                }
                const int ch = chb + (odd ? 16 : 0) + 8 * hi;
                if (ch < a.Nout) {
                    uint4 o0 = make_uint4(s0[0], s0[1], s0[2], s0[3]), o1 = make_uint4(s1[0], s1[1], s1[2], s1[3]);
                    if (ch + 7 >= a.Nout) {  // last chunk of a zero-padded tensor: zeros in its padding
                        const Mask8 k = make_mask8(a.Nout - ch);
                        o0 = mask8(o0, true, k);
                        o1 = mask8(o1, true, k);
                    }
                    if (ok0) *reinterpret_cast<uint4*>(a.D + dp0 + ch) = o0;
                    if (ok1) *reinterpret_cast<uint4*>(a.D + dp1 + ch) = o1;
                }
            }
        }
    } else {
        const int hi = lane >> 5;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int m = m0 + wm * WTM + tm * 32 + l32;
            int64_t dpix;
            int cell_h = 1, cell_w = 1;  // pixels of this lane's cell inside the destination image
            if (a.d_linear) {
                dpix = (int64_t)m * a.dpitch;
            } else {
                const uint32_t mm = (uint32_t)min(m, a.M - 1);
                const uint32_t row = fdiv(mm, a.gW), gj = mm - row * a.gW.d;
                const uint32_t n = fdiv(row, a.gH), gi = row - n * a.gH.d;
                const int dh = (int)gi * a.d_hmul + a.d_hadd, dw = (int)gj * a.d_wmul + a.d_wadd;
                dpix = (((int64_t)n * a.DH + dh) * a.DW + dw) * a.dpitch;
                cell_h = min(a.zf_h, a.DH - dh);
                cell_w = min(a.zf_w, a.DW - dw);
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int chb = n0 + wn * WTN + tn * 32;
                if (chb >= a.Nout) continue;  // wave-uniform
#pragma unroll
                for (int gp = 0; gp < 2; ++gp) {  // register pairs (g = 2gp, 2gp + 1)
                    const f32x16& c = acc[tn][tm];
                    const uint32_t p0 = cvt_pk_bf16(c[8 * gp + 0], c[8 * gp + 1]), q0 = cvt_pk_bf16(c[8 * gp + 2], c[8 * gp + 3]);
                    const uint32_t p1 = cvt_pk_bf16(c[8 * gp + 4], c[8 * gp + 5]), q1 = cvt_pk_bf16(c[8 * gp + 6], c[8 * gp + 7]);
                    const auto ps = __builtin_amdgcn_permlane32_swap(p0, p1, false, false);
                    const auto qs = __builtin_amdgcn_permlane32_swap(q0, q1, false, false);
                    const int ch = chb + 16 * gp + 8 * hi;
                    if (m < a.M && ch < a.Nout) {
                        uint16_t* dst = a.D + dpix + ch;
                        if (a.zf_h * a.zf_w > 1) {  // uniform: clear the other pixels of the cell (vector stores only)
                            for (int zh = 0; zh < cell_h; ++zh)
                                for (int zw = zh == 0 ? 1 : 0; zw < cell_w; ++zw)
                                    *reinterpret_cast<uint4*>(dst + ((int64_t)zh * a.DW + zw) * a.dpitch) = make_uint4(0u, 0u, 0u, 0u);
                        }
                        if (a.d_vec16 && ch + 7 < a.Nout) {
                            *reinterpret_cast<uint4*>(dst) = make_uint4(ps[0], qs[0], ps[1], qs[1]);
                        } else if (a.d_vec16 && a.pad_zero && ch + 8 <= a.dpitch) {
                            // zero-padded tensors: the last chunk goes out as one vector too, zeros in its padding
                            *reinterpret_cast<uint4*>(dst) =
                                mask8(make_uint4(ps[0], qs[0], ps[1], qs[1]), true, make_mask8(a.Nout - ch));
                        } else {
                            const uint32_t w[4] = {ps[0], qs[0], ps[1], qs[1]};
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (ch + e < a.Nout) dst[e] = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
                        }
                    }
                }
            }
        }
    }
    if constexpr (STATS) {
        // Every lane holds 16 channel values per 32x32 block (channels 8g + 4*(lane/32) + i, v = 4g + i) of one
        // pixel.  A halving butterfly over the 32 pixel lanes of each half-wave leaves lane l with the total of the
        // one value v(l) = bits (16, 8, 4, 2) of l: 16 exchanges per block and statistic instead of 80.
        float* red = reinterpret_cast<float*>(smem_b);  // [2][WGM][BN]; the stage buffers are dead after the barrier
        __syncthreads();
        const int hi = lane >> 5;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            float sv[16], qv[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) sv[v] = 0.f, qv[v] = 0.f;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const bool valid = m0 + wm * WTM + tm * 32 + l32 < a.M;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    // the value as stored: rounded to bf16
                    const float r = __uint_as_float(cvt_pk_bf16(acc[tn][tm][v], 0.f) << 16);
                    const float rv = valid ? r : 0.f;
                    sv[v] += rv;
                    qv[v] += rv * rv;
                }
            }
            static_for<0, 4>([&](auto step_c) {  // halves 8, 4, 2, 1 exchanged across lane bits 16, 8, 4, 2
                constexpr int HALF = 8 >> decltype(step_c)::value, BIT = 16 >> decltype(step_c)::value;
                const bool up = (l32 & BIT) != 0;
                static_for<0, HALF>([&](auto i_c) {
                    constexpr int I = decltype(i_c)::value;
                    const float ss = up ? sv[I] : sv[I + HALF], sq = up ? qv[I] : qv[I + HALF];
                    const float ks = up ? sv[I + HALF] : sv[I], kq = up ? qv[I + HALF] : qv[I];
                    sv[I] = ks + __shfl_xor(ss, BIT, 64);
                    qv[I] = kq + __shfl_xor(sq, BIT, 64);
                });
            });
            sv[0] += __shfl_xor(sv[0], 1, 64);
            qv[0] += __shfl_xor(qv[0], 1, 64);
            if ((l32 & 1) == 0) {
                const int v = ((l32 >> 4) & 1) * 8 + ((l32 >> 3) & 1) * 4 + ((l32 >> 2) & 1) * 2 + ((l32 >> 1) & 1);
                const int chl = wn * WTN + tn * 32 + 8 * (v >> 2) + 4 * hi + (v & 3);
                red[(0 * WGM + wm) * BN + chl] = sv[0];
                red[(1 * WGM + wm) * BN + chl] = qv[0];
            }
        }
        __syncthreads();
        const int tile_m = m0 / BM;
        for (int t = tid; t < 2 * BN; t += 64 * NW) {
            const int q = t / BN, chl = t - q * BN;
            if (n0 + chl >= a.Nout) continue;
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < WGM; ++w) tot += red[(q * WGM + w) * BN + chl];  // fixed order
            a.stats[((size_t)q * a.tiles_m + tile_m) * a.Nout + n0 + chl] = tot;
        }
    }
#endif
}

// What the host has decided for one problem of the direct kernel: which instantiation, and its launch shape.
typedef void (*igemm_dl_kern_t)(const IgemmArgsN);
struct IgemmDlPlan {
    igemm_dl_kern_t kern;
    LdsOptIn* opt_in;
    // the same instantiation with the tap validity tests (== kern unless the problem is free of them): what a group of
    // problems falls back to when only some of them could do without
    igemm_dl_kern_t kern_tests;
    LdsOptIn* opt_in_tests;
    size_t lds, lds_used;
    int threads;
};

// Problems that chose the same instantiation go out as ONE launch (blockIdx.y = problem): the tail of one overlaps the
// head of the next, and a group of short launches pays the fixed cost of a launch once.
inline hipError_t launch_igemm_dl_planned(const IgemmArgs* as, const IgemmDlPlan* ps, int n, hipStream_t st) {
    bool done[kIgemmMaxProblems] = {false, false, false, false};
    if (n > kIgemmMaxProblems) return hipErrorInvalidValue;
    IgemmDlPlan local[kIgemmMaxProblems];
    bool same = true, same_tests = true;
    for (int i = 1; i < n; ++i) {
        same = same && ps[i].kern == ps[0].kern;
        same_tests = same_tests && ps[i].kern_tests == ps[0].kern_tests;
    }
    if (!same && same_tests) {  // one launch with the validity tests rather than two without and with
        for (int i = 0; i < n; ++i) {
            local[i] = ps[i];
            local[i].kern = ps[i].kern_tests;
            local[i].opt_in = ps[i].opt_in_tests;
        }
        ps = local;
    }
    for (int i = 0; i < n; ++i) {
        if (done[i]) continue;
        IgemmArgsN m{};
        int cnt = 0, gx = 0;
        size_t lds_used = 0;
        for (int j = i; j < n; ++j) {
            if (done[j] || ps[j].kern != ps[i].kern) continue;
            done[j] = true;
            m.a[cnt++] = as[j];
            gx = as[j].grid_x > gx ? as[j].grid_x : gx;
            lds_used = ps[j].lds_used > lds_used ? ps[j].lds_used : lds_used;
        }
        if (hipError_t e = ps[i].opt_in->ensure(reinterpret_cast<const void*>(ps[i].kern), ps[i].lds); e != hipSuccess) return e;
        // (several problems: a width that is a multiple of the 8 XCDs keeps every problem's tile -> XCD assignment)
        const unsigned gxr = cnt > 1 ? (unsigned)((gx + 7) / 8 * 8) : (unsigned)gx;
        hipLaunchKernelGGL(ps[i].kern, dim3(gxr, (unsigned)cnt), dim3((unsigned)ps[i].threads), lds_used, st, m);
    }
    return hipSuccess;
}

template <int BM, int BN, int WGM, int WGN, int STAGES>
inline hipError_t plan_igemm_dl_cfg(IgemmArgs& a, IgemmDlPlan& plan) {
    constexpr int NT = 64 * WGM * WGN;
    constexpr size_t lds = (size_t)STAGES * (BM + BN) * 128;
    static_assert(lds <= 160 * 1024, "LDS capacity");
    // last channel block of a tap is short and/or some chunk has a masked tail
    const bool ragged = (a.Cred % 64) != 0 || (a.fold && a.Creal % 8 != 0);
    a.nk = a.TR * a.TS * (int)ceil_div(a.CredP, 64);  // steps are (tap, block of 64 channels)
    a.tiles_n = (int)ceil_div(a.Nout, BN);
    set_tail_tables(a);
    // variant: 0 = whole 64-channel blocks, 1 = partial blocks but no undefined elements (channel count a multiple
    // of 8, or the caller vouches for zero padding), 2 = partial blocks with tails to clear
    int variant = !ragged ? 0 : (a.tail_kv == 0 || a.pad_zero ? 1 : 2);
    if (a.stats) {  // statistics epilogue: variants 3, 4 = variants 0, 1 with it (the caller has ruled out tails)
        if (variant == 2) return hipErrorInvalidValue;
        variant += 3;
        a.tiles_m = (int)ceil_div(a.M, BM);
    }
    // buffer addressing of the gathered operand (see the kernel): shifts that make both address parts non-negative
    a.a_guard = ((a.h_add < 0 ? -a.h_add : 0) * a.srcW + (a.w_add < 0 ? -a.w_add : 0)) * a.apitch;
    const int last_r = (a.TR - 1) * a.tr_step, last_s = (a.TS - 1) * a.ts_step;
    a.a_smin = ((last_r < 0 ? last_r : 0) * a.srcW + (last_s < 0 ? last_s : 0)) * a.apitch;
    const int64_t img = (int64_t)ceil_div(a.M, (int64_t)a.gH.d * a.gW.d);  // images of the source tensor
    if ((img * a.srcH * a.srcW * a.apitch + a.a_guard) * 2 >= 0xffffff00ll) return hipErrorInvalidValue;
    if ((int64_t)a.Nout * a.b_taps * a.bpitch * 2 >= 0xffffff00ll) return hipErrorInvalidValue;
    // every tap of every row inside the source image?  coordinates are monotone in the grid index and in the tap
    auto inside = [](int lo, int hi, int n) { return lo >= 0 && hi >= 0 && lo < n && hi < n; };
    const int h_first = a.h_add, h_last = ((int)a.gH.d - 1) * a.h_mul + a.h_add;
    const int w_first = a.w_add, w_last = ((int)a.gW.d - 1) * a.w_mul + a.w_add;
    const int rr = (a.TR - 1) * a.tr_step, ss = (a.TSm - 1) * a.ts_step;
    a.a_all_valid = inside(h_first, h_last, a.srcH) && inside(h_first + rr, h_last + rr, a.srcH) &&
                    inside(w_first, w_last, a.srcW) && inside(w_first + ss, w_last + ss, a.srcW);
    const bool av = a.a_all_valid && variant != 2;
    typedef igemm_dl_kern_t kern_t;
    const kern_t kerns[2][5] = {{k_igemm_dl<BM, BN, WGM, WGN, STAGES, false, false, false, false>,
                                 k_igemm_dl<BM, BN, WGM, WGN, STAGES, true, false, false, false>,
                                 k_igemm_dl<BM, BN, WGM, WGN, STAGES, true, true, false, false>,
                                 k_igemm_dl<BM, BN, WGM, WGN, STAGES, false, false, true, false>,
                                 k_igemm_dl<BM, BN, WGM, WGN, STAGES, true, false, true, false>},
                                {k_igemm_dl<BM, BN, WGM, WGN, STAGES, false, false, false, true>,
                                 k_igemm_dl<BM, BN, WGM, WGN, STAGES, true, false, false, true>,
                                 nullptr,
                                 k_igemm_dl<BM, BN, WGM, WGN, STAGES, false, false, true, true>,
                                 k_igemm_dl<BM, BN, WGM, WGN, STAGES, true, false, true, true>}};
    static LdsOptIn opt_in[2][5];
    plan.kern = kerns[av ? 1 : 0][variant];
    plan.opt_in = &opt_in[av ? 1 : 0][variant];
    plan.kern_tests = kerns[0][variant];
    plan.opt_in_tests = &opt_in[0][variant];
    plan.lds = lds;
    plan.threads = NT;
    const int64_t tiles = ceil_div(a.M, BM) * a.tiles_n;
    if (tiles > 0x7fffffff) return hipErrorInvalidValue;
    a.grid_x = (int)tiles;
    // A reduction of fewer steps than the pipeline has stages touches only the first nk stage buffers (and the
    // statistics epilogue a few KB of the first): the launch asks for no more LDS than that, which leaves room on the
    // CU for workgroups of kernels running beside it (train step at pruned widths -0.6 %, full -0.2 %).
    plan.lds_used = (size_t)(a.nk < STAGES ? (a.nk < 1 ? 1 : a.nk) : STAGES) * (BM + BN) * 128;
    return hipSuccess;
}

template <int BM, int BN, int WGM, int WGN, int STAGES>
inline hipError_t launch_igemm_dl_cfg(IgemmArgs& a, hipStream_t st) {
    IgemmDlPlan plan;
    if (hipError_t e = plan_igemm_dl_cfg<BM, BN, WGM, WGN, STAGES>(a, plan); e != hipSuccess) return e;
    return launch_igemm_dl_planned(&a, &plan, 1, st);
}

// ------------------------------------------------------------------------------------------- //
// forward convolution of a network's first layer: image-like input, at most 4 channels at a pitch of 8
// ------------------------------------------------------------------------------------------- //
// The implicit-GEMM kernel treats such a layer as a GEMM over folded filter rows of S * 8 elements: 5 of every 8
// multiplied elements are padding, and every output pixel pulls R runs of S pixels from L2 into LDS again.  Here a
// workgroup walks over a run of tiles of 4 x 64 output pixels (x 64 output channels).  It keeps ALL its weights in
// registers for the whole run (a filter row is 8 taps x 4 channels = two 16-element MFMA steps; taps past S and
// channels past C are zero).  Per tile it loads the input patch under the tile ONCE, 8 bytes (4 channels) per pixel,
// into LDS in image order: the two taps a lane multiplies in one step are neighbouring pixels, 16 contiguous bytes, and
// consecutive output pixels read consecutive (stride 1) or every other (stride 2) such pair.  The patch of the next
// tile is fetched into registers before the current tile is multiplied and written to the other of two LDS buffers
// after it, so that its memory latency hides behind the MFMAs.  R * 2 MFMAs per 32 x 32 block: against the folded
// form half the matrix work and an eighth of the operand traffic.  Both operands' padding channels must be zero (the
// caller's PT_CONV_PAD_ZERO), the output takes 16-byte stores.
struct StemArgs {
    const uint16_t* X;   // [N][H][W][8]
    const uint16_t* Wt;  // [K][R][S][8]
    uint16_t* Y;         // [N][P][Q][ypitch]
    int N, H, W, P, Q, K, R, S, pad_h, pad_w, ypitch;
    int tiles_q, tiles_p;  // tiles per image along Q and P
    int tiles, run;        // N * tiles_p * tiles_q, and how many consecutive tiles one workgroup takes
};
constexpr int kStemTH = 4, kStemTW = 64, kStemMaxR = 8;
constexpr int kStemSlots = 512;  // 256 CUs x 2 resident workgroups

// RT: rows of the filter the multiply loop runs over (R itself, or 8 for any R <= 8: rows past R multiply zeros);
// NJ: 16-element steps per filter row (1 for S <= 4, else 2).
template <int STRIDE, int RT, int NJ>
__global__ __launch_bounds__(512, 4) void k_stem_fwd(const StemArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int PH = (kStemTH - 1) * STRIDE + RT;              // patch rows
    constexpr int PW = (kStemTW - 1) * STRIDE + 4 * NJ;          // patch columns: 4 taps per step
    constexpr int PWR = (PW + 1) & ~1;                           // row pitch in pixels: rows start on 16 bytes
    constexpr int PSZ = PH * PWR;
    __shared__ __attribute__((aligned(16))) uint2 patch[2][PSZ]; // [buffer][row][column], 4 channels each
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles_n = (a.K + 63) / 64;
    const int nt = blockIdx.x % tiles_n, chunk = blockIdx.x / tiles_n;
    const int n0 = nt * 64;
    const int first = chunk * a.run, last = first + a.run < a.tiles ? first + a.run : a.tiles;
    if (first >= last) return;  // whole workgroup
    const int ph_used = (kStemTH - 1) * STRIDE + a.R;            // rows of the patch this filter reaches (<= PH)

    // ---- weights -> registers: fragment (r, j) of this lane = taps 4j + 2h, 4j + 2h + 1 of filter row r, 4 channels each
    const int wm = wave & 3, wn = wave >> 2;      // tile row of this wave, half of the 64 output channels
    const int l32 = lane & 31, h = lane >> 5;
    const int n = n0 + wn * 32 + l32;             // output channel of this lane's weight rows
    const bool n_ok = n < a.K;
    bf16x8 wf[RT][NJ];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            uint2 lo = make_uint2(0u, 0u), hi = make_uint2(0u, 0u);
            const int s0 = 4 * j + 2 * h;
            if (n_ok && r < a.R) {
                const uint16_t* wr = a.Wt + ((int64_t)(n * a.R + r) * a.S) * 8;
                if (s0 < a.S) lo = *reinterpret_cast<const uint2*>(wr + s0 * 8);
                if (s0 + 1 < a.S) hi = *reinterpret_cast<const uint2*>(wr + (s0 + 1) * 8);
            }
            wf[r][j] = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
        }

    // ---- this thread's pixels of a patch: LDS slots tid + 512 * it, the same in every tile --------------------------
    // (their rows and columns are worked out again at every use, from a copy of the thread index that the compiler
    // cannot see through: kept across the tile loop they cost registers, which spill)
    constexpr int NLD = (PSZ + 511) / 512;
    uint2 pv[NLD];
    // All loads of a patch are issued back to back, as buffer loads on a descriptor of the tile's image: a pixel
    // outside the image, or in a row the filter does not reach, passes an offset past the descriptor's range and reads
    // zeros (no branch, no cleared register, so nothing the loads would have to wait for).
    constexpr uint32_t kBufOut = 0xffffffffu, kBufFlags = 0x00020000u;
    const uint32_t img_bytes = (uint32_t)(a.H * a.W) * 16u;
    auto fetch = [&](int tq, int tp, int img) {
        const int ih0 = tp * kStemTH * STRIDE - a.pad_h, iw0 = tq * kStemTW * STRIDE - a.pad_w;
        const __amdgpu_buffer_rsrc_t x_srd = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(a.X) + (int64_t)img * a.H * a.W * 8, 0, img_bytes, kBufFlags);
        int t0 = tid;
        asm volatile("" : "+v"(t0));
#pragma unroll
        for (int it = 0; it < NLD; ++it) {
            const int i = t0 + it * 512;
            const int prow = i / PWR, pcol = i - prow * PWR;
            const int ih = ih0 + prow, iw = iw0 + pcol;
            const bool ok = prow < ph_used && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;  // (rows >= PH: too)
            const auto got = __builtin_amdgcn_raw_buffer_load_b64(x_srd, ok ? (uint32_t)(ih * a.W + iw) * 16u : kBufOut, 0, 0);
            pv[it] = make_uint2(got[0], got[1]);
        }
    };
    auto park = [&](int buf) {
        int t0 = tid;
        asm volatile("" : "+v"(t0));
#pragma unroll
        for (int it = 0; it < NLD; ++it)
            if ((it + 1) * 512 <= PSZ || t0 + it * 512 < PSZ) patch[buf][t0 + it * 512] = pv[it];
    };
    // tiles are numbered (image, tile row, tile column), column fastest: the next one by counting up
    auto advance = [&](int& tq, int& tp, int& img) {
        if (++tq == a.tiles_q) {
            tq = 0;
            if (++tp == a.tiles_p) {
                tp = 0;
                ++img;
            }
        }
    };
    int ntq = first % a.tiles_q, ntp = (first / a.tiles_q) % a.tiles_p, nimg = first / (a.tiles_q * a.tiles_p);

    fetch(ntq, ntp, nimg);
    park(0);
    __syncthreads();
    const bool wave_n_live = n0 + wn * 32 < a.K;  // uniform
    // LDS element this lane's fragments start from: pixel l32 of the wave's tile row, tap 2h
    const int frag0 = wm * STRIDE * PWR + l32 * STRIDE + 2 * h;
    int buf = 0;
    for (int tile = first; tile < last; ++tile, buf ^= 1) {
        const bool more = tile + 1 < last;  // uniform
        const int tq = ntq, tp = ntp, img = nimg;
        advance(ntq, ntp, nimg);
        if (more) fetch(ntq, ntp, nimg);
        const int p = tp * kStemTH + wm, q0 = tq * kStemTW;
        const bool live = wave_n_live && p < a.P;  // uniform
        f32x16 acc[2];
        if (live) {
            // ---- multiply: this wave's 64 output pixels (tile row wm) x 32 output channels -------------------------
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[tm][v] = 0.f;
            const uint2* pb = patch[buf] + frag0;
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int tm = 0; tm < 2; ++tm) {
                        // taps 4j + 2h, 4j + 2h + 1 of filter row r under output pixel tm * 32 + l32: two neighbouring pixels
                        const uint2* src = pb + r * PWR + tm * 32 * STRIDE + 4 * j;
                        uint4 x4;
                        if constexpr (STRIDE == 2) {
                            x4 = *reinterpret_cast<const uint4*>(src);  // an even column: 16-byte aligned
                        } else {
                            const uint2 lo = src[0], hi = src[1];
                            x4 = make_uint4(lo.x, lo.y, hi.x, hi.y);
                        }
                        acc[tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[r][j], __builtin_bit_cast(bf16x8, x4), acc[tm], 0, 0, 0);
                    }
        }
        // The next patch goes to the other buffer (last read before the barrier that ended the previous tile) BEFORE this
        // tile's stores are issued: the wait for its loads then does not also wait for the stores behind them.
        if (more) park(buf ^ 1);
        if (live) {
            // ---- store: the lane-pair exchange of k_igemm_dl (64 contiguous bytes of 16 pixels per store instruction) ----
            // (a uniform base per tile and wave plus one 32-bit offset per lane; lane-derived values of this part are
            // worked out afresh per tile, not kept in registers across the multiply)
            const __amdgpu_buffer_rsrc_t y_srd = __builtin_amdgcn_make_buffer_rsrc(
                a.Y + ((int64_t)(img * a.P + p) * a.Q + q0) * a.ypitch + n0 + wn * 32, 0, 0xffffff00u, kBufFlags);
            int le = lane;
            asm volatile("" : "+v"(le));
            const int l32e = le & 31;
            const bool odd = (le & 1) != 0;
            const int chl = (odd ? 16 : 0) + 8 * (le >> 5);             // channel of this lane's chunk within the wave's 32
            const int ch = n0 + wn * 32 + chl;
#pragma unroll
            for (int tm = 0; tm < 2; ++tm) {
                const int q = q0 + tm * 32 + l32e;
                const uint32_t off0 = (uint32_t)((tm * 32 + (l32e & ~1)) * a.ypitch + chl) * 2u;  // pixel (q & ~1); (q | 1) is next
                const bool ok0 = (q & ~1) < a.Q, ok1 = (q | 1) < a.Q;
                const f32x16& c = acc[tm];
                uint32_t v[2][4];
#pragma unroll
                for (int gp = 0; gp < 2; ++gp) {
                    const uint32_t x0 = cvt_pk_bf16(c[8 * gp + 0], c[8 * gp + 1]), y0 = cvt_pk_bf16(c[8 * gp + 2], c[8 * gp + 3]);
                    const uint32_t x1 = cvt_pk_bf16(c[8 * gp + 4], c[8 * gp + 5]), y1 = cvt_pk_bf16(c[8 * gp + 6], c[8 * gp + 7]);
                    const auto ps = __builtin_amdgcn_permlane32_swap(x0, x1, false, false);
                    const auto qs = __builtin_amdgcn_permlane32_swap(y0, y1, false, false);
                    v[gp][0] = ps[0]; v[gp][1] = qs[0]; v[gp][2] = ps[1]; v[gp][3] = qs[1];
                }
                uint32_t s0[4], s1[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t give = odd ? v[0][e] : v[1][e];
                    const uint32_t got = (uint32_t)__shfl_xor((int)give, 1, 64);
                    s0[e] = odd ? got : v[0][e];
                    s1[e] = odd ? v[1][e] : got;
                }
                uint4 o0 = make_uint4(s0[0], s0[1], s0[2], s0[3]), o1 = make_uint4(s1[0], s1[1], s1[2], s1[3]);
                if (ch < a.K && ch + 7 >= a.K) {  // last chunk: zeros in its padding
                    const Mask8 k = make_mask8(a.K - ch);
                    o0 = mask8(o0, true, k);
                    o1 = mask8(o1, true, k);
                }
                // (a pixel past the row's end, a chunk past the channel count: an offset out of range, the store is dropped)
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o0), y_srd, ok0 && ch < a.K ? off0 : kBufOut, 0, 0);
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o1), y_srd,
                                                       ok1 && ch < a.K ? off0 + (uint32_t)a.ypitch * 2u : kBufOut, 0, 0);
            }
        }
        __syncthreads();
    }
#endif
}

// One run of tiles per workgroup slot of the chip (2 workgroups per CU): the weights are fetched once per run.
inline hipError_t launch_stem_fwd(StemArgs& a, int stride, int slots, hipStream_t st) {
    a.tiles_q = (a.Q + kStemTW - 1) / kStemTW;
    a.tiles_p = (a.P + kStemTH - 1) / kStemTH;
    const int64_t tiles = (int64_t)a.N * a.tiles_p * a.tiles_q;
    if (tiles <= 0) return hipSuccess;
    if (tiles > 0x3fffffff) return hipErrorInvalidValue;
    a.tiles = (int)tiles;
    a.run = (int)((tiles + slots - 1) / slots);
    const int64_t grid = ((tiles + a.run - 1) / a.run) * ((a.K + 63) / 64);
    if (grid > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 g((unsigned)grid), b(512);
    const int nj = a.S <= 4 ? 1 : 2;
#define PT_STEM_CASE(ST, RT, NJ) hipLaunchKernelGGL((k_stem_fwd<ST, RT, NJ>), g, b, 0, st, a)
    if (stride == 1) {
        if (a.R == 3 && nj == 1) PT_STEM_CASE(1, 3, 1);
        else if (a.R == 7 && nj == 2) PT_STEM_CASE(1, 7, 2);
        else PT_STEM_CASE(1, 8, 2);
    } else {
        if (a.R == 3 && nj == 1) PT_STEM_CASE(2, 3, 1);
        else if (a.R == 7 && nj == 2) PT_STEM_CASE(2, 7, 2);
        else PT_STEM_CASE(2, 8, 2);
    }
#undef PT_STEM_CASE
    return hipSuccess;
}

// ------------------------------------------------------------------------------------------- //
// weight gradient
// ------------------------------------------------------------------------------------------- //
struct WgradArgs {
    const uint16_t* X;   // x[N][H][W][xpitch]
    const uint16_t* DY;  // dy[pixels][ypitch]
    float* OUT;          // splits > 1: partial[split][K][Mtot]; else dw[K][RS][wpitch]
    int pixels;          // N*P*Q
    FastDiv Q, P;
    int H, W, xpitch, ypitch;
    int stride_h, stride_w, pad_h, pad_w;
    int S, RS, C, CP;    // CP = C rounded up to 8; Mtot = RS*CP
    int Mtot, K;
    int tiles_n;         // tiles along K
    int tiles_m;         // tiles along (tap, c)
    int tiles_per_tap;   // direct kernel: channel blocks per filter tap
    int KP;              // K rounded up to 8
    int fold;            // direct kernel: a tile row block spans the S taps of one filter row (dense small-C pixels)
    int iters_total, iters_per_split, splits;
    int dn, dp, dq;      // direct kernel: one reduction step of BKP pixels = dn images + dp output rows + dq output columns
    int affine;          // direct kernel: stride 1 and output grid == input grid: x sits at (pixel + tap shift) * xpitch
    int x_all_valid;     // affine and no tap ever leaves the image (1 x 1 filter without padding)
    // direct kernel writing dw itself (direct != 0): when lw is set, the gradient of the group-lasso penalty is added
    // to every element on the way out, dw += l_lambda * (lw * (1/l_on[k] + 1/l_in[c])) with a zero norm contributing 0
    const float* lw;    // fp32 master weights, layout and pitch of dw
    const float* l_on;  // [K], nullptr = output groups not regularised
    const float* l_in;  // [C], nullptr = input groups not regularised
    float l_lambda;
    int out_row_pitch;   // elements between consecutive k in the partial buffer (Mtot)
    int wpitch;
    int direct;          // 1: write dw layout directly (splits == 1)
    int o_vec;
};

template <int BM, int BN, int BK, int WGM, int WGN, int MINB, bool VEC>
__global__ __launch_bounds__(64 * WGM * WGN, MINB) void k_wgrad(const WgradArgs a) {
    // LDS tiles are [pixel][channel] with a row pad of 32 elements (64 bytes): the four pixel rows a
    // 16-lane group touches in one transpose read then fall into different banks.
    constexpr int NT = 64 * WGM * WGN;
    constexpr int LDM = BM + 32, LDN = BN + 32;
    constexpr int XV = BM / 8, YV = BN / 8;  // 8-vectors per pixel row
    constexpr int XR = NT / XV, YR = NT / YV;  // pixel rows per pass
    constexpr int XP = BK / XR, YP = BK / YR;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int STAGE_ELEMS = BK * (LDM + LDN);
    static_assert(XP >= 1 && YP >= 1 && TM >= 1 && TN >= 1 && BK % 16 == 0 && BK % XR == 0 && BK % YR == 0, "tile config");
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction
    // Workgroup ids are dealt round-robin to the 8 XCDs.  All tiles of one pixel split read the same x and dy
    // slabs, so each XCD gets a contiguous range of the split-major (split, tile) order: a split's tiles run
    // back to back on one XCD and the slabs are fetched into that L2 once.
    const int ntile = a.tiles_m * a.tiles_n;
    const int lin = xcd_remap(blockIdx.x, gridDim.x);
    const int split = lin / ntile;
    const int tile = lin - split * ntile;
    const int n0 = (tile % a.tiles_n) * BN;  // k origin
    const int m0 = (tile / a.tiles_n) * BM;  // (tap, c) origin
    const int it0 = split * a.iters_per_split;
    const int it1 = min(a.iters_total, it0 + a.iters_per_split);

    // ---- loader state: every thread keeps one fixed 8-channel column of each tile ---------------
    const int xcv = tid % XV, xrow = tid / XV;
    const int mrow0 = m0 + xcv * 8;
    const int tap = mrow0 / a.CP, xc0 = mrow0 - tap * a.CP;
    const int fr = tap / a.S, fs = tap - fr * a.S;
    const int x_nvalid = (tap < a.RS) ? a.C - xc0 : 0;
    const int ycv = tid % YV, yrow = tid / YV;
    const int yk0 = n0 + ycv * 8;
    const int y_nvalid = a.K - yk0;

    const Mask8 xmask = make_mask8(x_nvalid), ymask = make_mask8(y_nvalid);
    uint4 rx[XP], ry[YP];
    bool okx[XP], oky[YP];
    auto gload = [&](int it) {
        const int pbase = it * BK;
#pragma unroll
        for (int i = 0; i < XP; ++i) {
            const int pix = pbase + xrow + i * XR;
            const uint32_t row = fdiv((uint32_t)pix, a.Q);
            const int q = pix - (int)row * (int)a.Q.d;
            const uint32_t n = fdiv(row, a.P);
            const int p = (int)row - (int)n * (int)a.P.d;
            const int ih = p * a.stride_h - a.pad_h + fr, iw = q * a.stride_w - a.pad_w + fs;
            okx[i] = pix < a.pixels && x_nvalid > 0 && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            const uint32_t off = (uint32_t)(((int)n * a.H + ih) * a.W + iw) * (uint32_t)a.xpitch + (uint32_t)xc0;
            rx[i] = ldg8<VEC>(a.X, okx[i] ? off : 0u, x_nvalid);
        }
#pragma unroll
        for (int i = 0; i < YP; ++i) {
            const int pix = pbase + yrow + i * YR;
            oky[i] = pix < a.pixels && y_nvalid > 0;
            ry[i] = ldg8<VEC>(a.DY, oky[i] ? (uint32_t)pix * (uint32_t)a.ypitch + (uint32_t)yk0 : 0u, y_nvalid);
        }
    };
    auto sstore = [&](int buf) {
        uint16_t* sX = smem + buf * STAGE_ELEMS;
        uint16_t* sY = sX + BK * LDM;
#pragma unroll
        for (int i = 0; i < XP; ++i)
            *reinterpret_cast<uint4*>(&sX[(xrow + i * XR) * LDM + xcv * 8]) = mask8(rx[i], okx[i], xmask);
#pragma unroll
        for (int i = 0; i < YP; ++i)
            *reinterpret_cast<uint4*>(&sY[(yrow + i * YR) * LDN + ycv * 8]) = mask8(ry[i], oky[i], ymask);
    };

    // ---- MFMA state ---------------------------------------------------------------------------
    const int wm = wave % WGM, wn = wave / WGM;
    // transpose-read geometry: 16-lane group g, lane t in group; source lane t points at pixel row
    // (t/4) and channel quad (t%4); the result is 4 consecutive pixels for channel 16*(g&1) + t.
    const int g16 = lane >> 4, t16 = lane & 15;
    const int tr_row = (g16 >> 1) * 8 + (t16 >> 2);     // + 4*h + ks*16
    const int tr_col = (g16 & 1) * 16 + (t16 & 3) * 4;  // + block origin
    f32x16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;
    bool m_live[TM], n_live[TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) m_live[tm] = m0 + wm * WTM + tm * 32 < a.Mtot;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) n_live[tn] = n0 + wn * WTN + tn * 32 < a.K;

    auto tr_read = [&](const uint16_t* base, int ld, int row, int col) -> bf16x8 {
        typedef __attribute__((address_space(3))) s16x4* lds_p;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(base + row * ld + col));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(base + (row + 4) * ld + col));
        s16x8 r;
        r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
        r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
        return __builtin_bit_cast(bf16x8, r);
    };

    if (it0 < it1) {
        gload(it0);
        sstore(0);
    }
    __syncthreads();
    bool all_live = true;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) all_live = all_live && m_live[tm];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) all_live = all_live && n_live[tn];
    auto compute = [&](int buf, auto check_tag) {
        constexpr bool CHECK = decltype(check_tag)::value;
        const uint16_t* sX = smem + buf * STAGE_ELEMS;
        const uint16_t* sY = sX + BK * LDM;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fx[TM], fy[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) fx[tm] = tr_read(sX, LDM, ks * 16 + tr_row, wm * WTM + tm * 32 + tr_col);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) fy[tn] = tr_read(sY, LDN, ks * 16 + tr_row, wn * WTN + tn * 32 + tr_col);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    if (!CHECK || (m_live[tm] && n_live[tn]))
                        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[tm], fy[tn], acc[tm][tn], 0, 0, 0);
        }
    };
    auto main_loop = [&](auto check_tag) {
        for (int it = it0; it < it1; ++it) {
            const int buf = (it - it0) & 1;
            if (it + 1 < it1) gload(it + 1);
            compute(buf, check_tag);
            if (it + 1 < it1) sstore(buf ^ 1);
            __syncthreads();
        }
    };
    if (all_live) main_loop(std::false_type{});
    else main_loop(std::true_type{});

    // ---- epilogue: lane holds k (column) = lane%32 and rows 8g + 4*(lane/32) + {0..3} = 4 consecutive c
    float* out = a.OUT + (a.direct ? 0 : (int64_t)split * a.K * a.out_row_pitch);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int k = n0 + wn * WTN + tn * 32 + (lane & 31);
        if (k >= a.K) continue;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int mrow = m0 + wm * WTM + tm * 32 + 8 * g + (lane >> 5) * 4;
                if (mrow >= a.Mtot) continue;
                const float v0 = acc[tm][tn][4 * g + 0], v1 = acc[tm][tn][4 * g + 1];
                const float v2 = acc[tm][tn][4 * g + 2], v3 = acc[tm][tn][4 * g + 3];
                if (a.direct) {
                    const int tp = mrow / a.CP, c = mrow - tp * a.CP;  // 4 consecutive rows share a tap (CP % 8 == 0)
                    float* dst = out + ((int64_t)k * a.RS + tp) * a.wpitch + c;
                    if (a.o_vec && c + 3 < a.C) {
                        *reinterpret_cast<float4*>(dst) = make_float4(v0, v1, v2, v3);
                    } else {
                        if (c < a.C) dst[0] = v0;
                        if (c + 1 < a.C) dst[1] = v1;
                        if (c + 2 < a.C) dst[2] = v2;
                        if (c + 3 < a.C) dst[3] = v3;
                    }
                } else {
                    *reinterpret_cast<float4*>(out + (int64_t)k * a.out_row_pitch + mrow) = make_float4(v0, v1, v2, v3);
                }
            }
        }
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, int MINB, bool VEC = true>
inline hipError_t launch_wgrad_cfg(WgradArgs& a, hipStream_t st) {
    constexpr int NT = 64 * WGM * WGN;
    constexpr size_t lds = (size_t)2 * BK * (BM + 32 + BN + 32) * 2;
    auto kern = k_wgrad<BM, BN, BK, WGM, WGN, MINB, VEC>;
    static LdsOptIn opt_in;
    if (hipError_t e = opt_in.ensure(reinterpret_cast<const void*>(kern), lds); e != hipSuccess) return e;
    a.tiles_m = (int)ceil_div(a.Mtot, BM);
    a.tiles_n = (int)ceil_div(a.K, BN);
    hipLaunchKernelGGL(kern, dim3(a.tiles_m * a.tiles_n * a.splits), dim3(NT), lds, st, a);
    return hipSuccess;
}

// ------------------------------------------------------------------------------------------- //
// weight gradient with direct global->LDS loads (vector path)
// ------------------------------------------------------------------------------------------- //
// Output tile: BM input channels of ONE filter tap x BN output channels; reduction over output pixels
// in steps of BKP.  Both tiles are pixel-major in LDS exactly as they sit in memory (a pixel row of
// the x tile is BM channels = 2*BM bytes), filled by 16-byte global->LDS loads and read back with the
// transpose read.  The 32-byte units of a row are permuted with the pixel row (see unit_phys in the kernel) so that
// the eight units the first and the second half-wave touch in one transpose read fall into different banks.  Pixels
// whose tap falls outside the image, and pixels past the end, are fetched as zeros (an out-of-range buffer offset, or
// the zero page in the general gather; both operands, so no garbage ever meets a zero).  Channel chunks past the channel count re-read the last valid chunk:
// they only feed accumulator rows/columns that are never stored.
// Transposing LDS read issued as inline assembly.  The compiler cannot see which LDS bytes the intrinsic
// form touches and therefore waits for every outstanding global->LDS load before it, which serialises the
// software pipeline; issued this way the read is ordered only by the explicit waits below.  The result
// registers must not be touched before lds_wait() has been applied to them.
template <int OFF>
__device__ __forceinline__ s16x4 lds_read_tr16_b64(uint32_t addr) {
    static_assert(OFF >= 0 && OFF < 65536, "DS offset field");
    s16x4 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
__device__ __forceinline__ bf16x8 join_halves(s16x4 lo, s16x4 hi) {
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// KSPLIT wave groups share one tile: group g multiplies the g-th part of every stage's pixel sub-steps, and the
// groups' accumulators are added through LDS before the store.  More waves per SIMD to hide LDS and barrier
// latency, with the same LDS footprint, loads and partial-sum traffic as one group.
// XMODE: how x is addressed.  0 = any geometry (per-lane global addresses, advanced incrementally); 1 = stride 1 with
// an output grid equal to the input grid ('same'-padded filters): buffer loads whose moving part is a scalar; 2 = the
// same where no tap ever leaves the image (1 x 1 filters): no per-lane work at all in a reduction step.
template <int BM, int BN, int BKP, int WGM, int WGN, int STAGES, int KSPLIT = 1, int MINB = 1, int XMODE = 0>
__global__ __launch_bounds__(64 * WGM * WGN * KSPLIT, MINB) void k_wgrad_dl(const WgradArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub
    constexpr int NWT = WGM * WGN;       // waves of one group: the wave grid over the tile
    constexpr int NW = NWT * KSPLIT;     // all waves: they share the loads
    constexpr int RBX = BM * 2, RBY = BN * 2;              // bytes per pixel row
    constexpr int CPRX = RBX / 16, CPRY = RBY / 16;        // 16-byte chunks per row
    constexpr int RPLX = 64 / CPRX, RPLY = 64 / CPRY;      // pixel rows per wave-level load
    constexpr int LX = BKP / RPLX / NW, LY = BKP / RPLY / NW;  // loads per lane per stage
    constexpr int LPT = LX + LY;
    constexpr int XBYTES = BKP * RBX, STAGE_BYTES = BKP * (RBX + RBY);
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert((RBX == 128 || RBX == 256) && (RBY == 128 || RBY == 256), "row size");
    static_assert(NW % 2 == 0 && LX >= 1 && LY >= 1 && BKP % (RPLX * NW) == 0 && BKP % (RPLY * NW) == 0, "tile config");
    static_assert(TM >= 1 && TN >= 1 && BKP % 16 == 0 && STAGES >= 2 && (STAGES - 2) * LPT < 64, "tile config");
    static_assert(KSPLIT >= 1 && (BKP / 16) % KSPLIT == 0 && NW <= 16, "wave groups");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_b[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = wave / NWT, wave_t = wave - kg * NWT;  // wave group, wave inside the group
    // Workgroup ids are dealt round-robin to the 8 XCDs.  All tiles of one pixel split read the same x and dy
    // slabs, so each XCD gets a contiguous range of the split-major (split, tile) order: a split's tiles run
    // back to back on one XCD and the slabs are fetched into that L2 once.
    const int ntile = a.tiles_m * a.tiles_n;
    const int lin = xcd_remap(blockIdx.x, gridDim.x);
    const int split = lin / ntile;
    const int tile = lin - split * ntile;
    const int n0 = (tile % a.tiles_n) * BN;        // k origin
    const int mt = tile / a.tiles_n;               // (tap, channel block)
    // tile row block: one filter tap (CP channels), or in folded mode one filter row (S*CP contiguous elements)
    const int tb = mt / a.tiles_per_tap;
    const int cb = (mt - tb * a.tiles_per_tap) * BM;
    const int run = a.fold ? a.S * a.CP : a.CP;
    const int fr = a.fold ? tb : tb / a.S;
    const int it0 = split * a.iters_per_split;
    const int it1 = min(a.iters_total, it0 + a.iters_per_split);

    // Placement of the 32-byte units (16 channels) of a pixel row, constant per lane over its loads.  A transposing
    // read takes, per 16-lane group, one unit from each of four consecutive pixel rows, and the LDS serves two such
    // groups per cycle (64 banks of 4 bytes): lanes 0-31 read units u and u + 1 (u even) of the same four rows, lanes
    // 32-63 the same of rows + 8.  So the low bit of the logical unit becomes the high bit of the physical one (u and
    // u + 1 land in different halves of a 256-byte bank line) and the remaining bits are XOR-ed with the row so that
    // the four rows of a group differ: 2.5 instead of 4.1 cycles per read against XOR-ing all bits with the row.
    // 128-byte rows: consecutive rows already alternate between the halves of a bank line.
    auto unit_phys = [](int u, int row, int rb) {
        return rb == 256 ? (((u >> 1) | ((u & 1) << 2)) ^ (row & 3)) : ((((u & 1) << 1) | (u >> 1)) ^ ((row >> 1) & 1));
    };
    auto unit_logical = [](int p, int row, int rb) {  // inverse of unit_phys in u
        if (rb == 256) {
            const int q = p ^ (row & 3);
            return ((q & 3) << 1) | (q >> 2);
        }
        const int q = p ^ ((row >> 1) & 1);
        return ((q & 1) << 1) | (q >> 1);
    };
    // x tile: this lane's row inside a wave-level load, and the logical 8-channel chunk it fetches
    const int xr = lane / CPRX, xpc = lane % CPRX;
    const int xlc = (unit_logical(xpc >> 1, wave * RPLX + xr, RBX) << 1) | (xpc & 1);
    const int xc = min(cb + xlc * 8, run - 8);     // clamp: chunks past the run are never stored
    const int fs = a.fold ? xc / a.CP : tb - fr * a.S;   // filter column of this lane's chunk
    const int fs_addr = a.fold ? 0 : fs;           // folded: the column offset is part of xc
    const int yr = lane / CPRY, ypc = lane % CPRY;
    const int ylc = (unit_logical(ypc >> 1, wave * RPLY + yr, RBY) << 1) | (ypc & 1);
    const int yk = min(n0 + ylc * 8, a.KP - 8);
    const uint16_t* zero_page = reinterpret_cast<const uint16_t*>(g_zero16);

    // Gather state of this lane's loads, advanced by BKP pixels per reduction step without divisions or multiplies
    // (integer multiplies run at a quarter of the vector rate and were the loop's bound).  A step moves every
    // slot from output pixel (n, p, q) to (n + dn, p + dp, q + dq) with at most one carry out of q and one out of
    // p (dq < Q, dp < P); the slot keeps the input coordinates (ih, iw) of its tap and the element offset of that
    // input pixel, which change by constants that depend only on the two carries.
    const int Qs = (int)a.Q.d * a.stride_w, Ps = (int)a.P.d * a.stride_h;
    const int iw_wrap = Qs - a.pad_w + fs, ih_wrap = Ps - a.pad_h + fr;  // first coordinate past the last output column / row
    const int dq_s = a.dq * a.stride_w, dp_s = a.dp * a.stride_h;
    const int rowp = a.W * a.xpitch;  // elements per input row
    const int D0 = dq_s * a.xpitch + dp_s * rowp + a.dn * a.H * rowp;  // no carry
    const int D1 = a.stride_h * rowp - Qs * a.xpitch;                  // carry out of q: next output row
    const int D2 = (a.H - Ps) * rowp;                                  // carry out of p: next image
    const int xrel0 = wave * RPLX + xr, yrel0 = wave * RPLY + yr;      // this lane's pixel inside a step (slot 0)
    int x_ih[LX], x_iw[LX];
    uint32_t x_off[LX];
#pragma unroll
    for (int j = 0; j < LX; ++j) {
        const int pix = it0 * BKP + xrel0 + NW * j * RPLX;
        const uint32_t row = fdiv((uint32_t)pix, a.Q);
        const int q = pix - (int)row * (int)a.Q.d;
        const uint32_t n = fdiv(row, a.P);
        const int p = (int)row - (int)n * (int)a.P.d;
        x_ih[j] = p * a.stride_h - a.pad_h + fr;
        x_iw[j] = q * a.stride_w - a.pad_w + fs;
        x_off[j] = (uint32_t)(((int)n * a.H + x_ih[j]) * a.W + (x_iw[j] - fs + fs_addr)) * (uint32_t)a.xpitch + (uint32_t)xc;
    }
    // pixels from the next step's first one to the end of this workgroup's slice (uniform): loads past it fetch zeros,
    // so steps may be issued unconditionally
    int p_left = min(a.pixels, it1 * BKP) - it0 * BKP;

    // dy, and x in layers whose output grid equals the input grid at stride 1 (1x1 and 'same'-padded filters), sit at
    // an address that is affine in the output pixel index: a reduction step moves every load by one uniform amount.
    // Those loads are buffer loads: the per-lane part of the address is a constant (voffset), the moving part a
    // scalar register (soffset), and a lane that must read zeros (tap outside the image, pixel past the end) passes
    // an out-of-range voffset, for which the load writes zeros to LDS.  The loop is bound by the number of
    // instructions a wave issues per step, so nothing is computed per lane and step beyond the validity of
    // 'same'-padded taps.  The filter tap's shift is folded into the buffer's base address (it may point ahead of the
    // tensor: only valid taps are ever fetched).
    constexpr uint32_t kBufRecords = 0x40000000u, kBufOut = 0x80000000u, kBufFlags = 0x00020000u;
    const int tapshift = XMODE ? ((fr - a.pad_h) * a.W + (fs_addr - a.pad_w)) * a.xpitch : 0;  // uniform
    const __amdgpu_buffer_rsrc_t x_srd =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.X) + tapshift, 0, kBufRecords, kBufFlags);
    const __amdgpu_buffer_rsrc_t y_srd = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.DY), 0, kBufRecords, kBufFlags);
    const uint32_t x_v = (uint32_t)(xr * a.xpitch + xc) * 2u, y_v = (uint32_t)(yr * a.ypitch + yk) * 2u;  // bytes
    uint32_t x_s[LX], y_s[LY];  // scalar byte offsets of the slots' pixel rows
#pragma unroll
    for (int j = 0; j < LX; ++j) x_s[j] = (uint32_t)(it0 * BKP + (wave + NW * j) * RPLX) * (uint32_t)a.xpitch * 2u;
#pragma unroll
    for (int j = 0; j < LY; ++j) y_s[j] = (uint32_t)(it0 * BKP + (wave + NW * j) * RPLY) * (uint32_t)a.ypitch * 2u;
    const uint32_t x_step = (uint32_t)(BKP * a.xpitch) * 2u, y_step = (uint32_t)(BKP * a.ypitch) * 2u;

    // issues the loads of the next reduction step (steps are issued in order) into `stage`
    auto issue = [&](int stage) {
        uint8_t* sbase = smem_b + stage * STAGE_BYTES;
        const bool whole = p_left >= BKP;  // uniform: every pixel of the step lies inside the slice
        if constexpr (XMODE == 0) {
#pragma unroll
            for (int j = 0; j < LX; ++j) {
                const bool ok = xrel0 < p_left - NW * j * RPLX && (unsigned)x_ih[j] < (unsigned)a.H && (unsigned)x_iw[j] < (unsigned)a.W;
                __builtin_amdgcn_global_load_lds(pick_ptr(ok, a.X + x_off[j], zero_page),
                                                 (lds_void_ptr)(sbase + (wave + NW * j) * 1024), 16, 0, 0);
                const int iw = x_iw[j] + dq_s;
                const bool c1 = iw >= iw_wrap;
                x_iw[j] = iw - (c1 ? Qs : 0);
                const int ih = x_ih[j] + (c1 ? dp_s + a.stride_h : dp_s);
                const bool c2 = ih >= ih_wrap;
                x_ih[j] = ih - (c2 ? Ps : 0);
                x_off[j] += (uint32_t)((c1 ? D0 + D1 : D0) + (c2 ? D2 : 0));
            }
        } else {
            uint32_t v[LX];
#pragma unroll
            for (int j = 0; j < LX; ++j) {
                v[j] = x_v;
                if constexpr (XMODE == 1) {
                    const bool ok = (unsigned)x_ih[j] < (unsigned)a.H && (unsigned)x_iw[j] < (unsigned)a.W;
                    v[j] = ok ? x_v : kBufOut;
                    const int iw = x_iw[j] + dq_s;
                    const bool c1 = iw >= iw_wrap;
                    x_iw[j] = iw - (c1 ? Qs : 0);
                    const int ih = x_ih[j] + (c1 ? dp_s + 1 : dp_s);
                    x_ih[j] = ih - (ih >= ih_wrap ? Ps : 0);
                }
            }
            if (!whole) {
#pragma unroll
                for (int j = 0; j < LX; ++j) v[j] = xrel0 < p_left - NW * j * RPLX ? v[j] : kBufOut;
            }
#pragma unroll
            for (int j = 0; j < LX; ++j) {
                __builtin_amdgcn_raw_ptr_buffer_load_lds(x_srd, (lds_void_ptr)(sbase + (wave + NW * j) * 1024), 16, v[j], x_s[j], 0, 0);
                x_s[j] += x_step;
            }
        }
        uint32_t vy[LY];
#pragma unroll
        for (int j = 0; j < LY; ++j) vy[j] = y_v;
        if (!whole) {
#pragma unroll
            for (int j = 0; j < LY; ++j) vy[j] = yrel0 < p_left - NW * j * RPLY ? y_v : kBufOut;
        }
#pragma unroll
        for (int j = 0; j < LY; ++j) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(y_srd, (lds_void_ptr)(sbase + XBYTES + (wave + NW * j) * 1024), 16, vy[j], y_s[j], 0, 0);
            y_s[j] += y_step;
        }
        p_left -= BKP;
    };

    // ---- MFMA state ---------------------------------------------------------------------------
    const int wm = wave_t % WGM, wn = wave_t / WGM;
    // transpose-read geometry: 16-lane group g16, lane t16; source lane t16 points at pixel row (t16 >> 2)
    // and channel quad (t16 & 3); the result is 4 consecutive pixels for channel 16*(g16 & 1) + t16.
    const int g16 = lane >> 4, t16 = lane & 15;
    const int tr_row = (g16 >> 1) * 8 + (t16 >> 2);  // + 4*h + ks*16
    const int tr_u = (g16 & 1);                       // 16-channel unit inside a 32-channel block
    const int tr_b = (t16 & 3) * 8;                   // byte inside the unit
    f32x16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

    // 32-bit LDS addresses of this lane's transposing reads: per 32-wide tile the 4-pixel halves at rows r, r+4.
    // The swizzle term does not depend on the 16-pixel sub-step, which therefore is an immediate offset.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_ptr)smem_b;
    constexpr int NKS = BKP / 16 / KSPLIT, NRD = 2 * (TM + TN);  // sub-steps per stage and group, LDS reads per sub-step
    uint32_t ax[TM][2], ay[TN][2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int r = tr_row + 4 * h;
        const int r0 = kg * NKS * 16;  // first pixel row of this group's sub-steps (a multiple of 16: same swizzle)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int u = (wm * WTM + tm * 32) / 16 + tr_u;
            ax[tm][h] = lds_base + (uint32_t)((r0 + r) * RBX + (unit_phys(u, r, RBX) << 5) + tr_b);
        }
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int u = (wn * WTN + tn * 32) / 16 + tr_u;
            ay[tn][h] = lds_base + (uint32_t)((r0 + r) * RBY + (unit_phys(u, r, RBY) << 5) + tr_b);
        }
    }
    static_assert(NKS == 1 || NRD < 16, "fragment reads per sub-step must fit the lgkmcnt field");
    // One stage: the reads of sub-step ks+1 are in flight while the MFMAs of sub-step ks run.
    auto compute = [&](int stage) {
        const uint32_t sb = (uint32_t)(stage * STAGE_BYTES);
        s16x4 fx[2][TM][2], fy[2][TN][2];
        auto issue_reads = [&](auto ks_c) {
            constexpr int KS = decltype(ks_c)::value;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int h = 0; h < 2; ++h) fx[KS & 1][tm][h] = lds_read_tr16_b64<KS * 16 * RBX>(ax[tm][h] + sb);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int h = 0; h < 2; ++h) fy[KS & 1][tn][h] = lds_read_tr16_b64<XBYTES + KS * 16 * RBY>(ay[tn][h] + sb);
        };
        issue_reads(std::integral_constant<int, 0>{});
        static_for<0, NKS>([&](auto ks_c) {
            constexpr int KS = decltype(ks_c)::value, B = KS & 1;
            if constexpr (KS + 1 < NKS) {
                issue_reads(std::integral_constant<int, KS + 1>{});
                lds_wait<NRD>(fx[B][0][0]);
            } else {
                lds_wait<0>(fx[B][0][0]);
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int h = 0; h < 2; ++h) lds_tie(fx[B][tm][h]);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int h = 0; h < 2; ++h) lds_tie(fy[B][tn][h]);
            bf16x8 vx[TM], vy[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) vx[tm] = join_halves(fx[B][tm][0], fx[B][tm][1]);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) vy[tn] = join_halves(fy[B][tn][0], fy[B][tn][1]);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vy[tn], vx[tm], acc[tm][tn], 0, 0, 0);
            // keep this sub-step's MFMAs ahead of the next sub-step's wait: otherwise the scheduler sinks them below
            // it and nothing overlaps the fragment reads
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    const int nk = it1 - it0;
    const bool late = STAGES >= 3 && NW >= 8 && (wave & 4) != 0;
    // Loads run STAGES - 1 steps ahead and are issued at every step, also past the slice's end (they then fetch
    // zeros into a stage nobody reads): the number of loads in flight is the same at every wait.
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue(s);
    for (int kt0 = 0; kt0 < nk; kt0 += STAGES) {
#pragma unroll
        for (int s = 0; s < STAGES; ++s) {
            if (kt0 + s < nk) {
                wait_vmcnt<(STAGES - 2) * LPT>();
                barrier_nofence();
                // Waves w and w+4 share a SIMD.  With three or more stages one of them issues the next stage's
                // loads before its MFMAs and the other after, so the two phases overlap on the SIMD instead of
                // running in lockstep.  The target buffer is the one consumed in the previous step either way.
                if (!late) issue((s + STAGES - 1) % STAGES);
                compute(s);
                if (late) issue((s + STAGES - 1) % STAGES);
            }
        }
    }
    wait_vmcnt<0>();  // the loads issued past the end have landed before LDS is reused or the wave ends

    if constexpr (KSPLIT > 1) {
        // groups 1.. park their accumulators in LDS one group at a time (the stage buffers are dead: every load was
        // waited for and the barrier below follows every wave's last read); group 0 adds them in group order and stores
        float* red = reinterpret_cast<float*>(smem_b);
        constexpr int PER_WAVE = TM * TN * 16 * 64;
#pragma unroll
        for (int g = 1; g < KSPLIT; ++g) {
            __syncthreads();
            if (kg == g) {
                float* dst = red + wave_t * PER_WAVE + lane;
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int v = 0; v < 16; ++v) dst[((tm * TN + tn) * 16 + v) * 64] = acc[tm][tn][v];
            }
            __syncthreads();
            if (kg == 0) {
                const float* src = red + wave_t * PER_WAVE + lane;
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[tm][tn][v] += src[((tm * TN + tn) * 16 + v) * 64];
            }
        }
        if (kg > 0) return;
    }
    // ---- epilogue: the MFMA's row operand is dy, so a lane holds input channel (column) lane%32 of the 32x32 block
    // and output channels (rows) 8g + 4*(lane/32) + {0..3}: a store instruction writes, for one output channel per
    // half-wave, 32 consecutive input channels = 128 contiguous bytes of dw (or of the partial slab).
    float* out = a.OUT + (a.direct ? 0 : (int64_t)split * a.K * a.out_row_pitch);
    const int hi4 = (lane >> 5) * 4;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int cr = cb + wm * WTM + tm * 32 + (lane & 31);  // row inside the run
        if (cr >= run) continue;
        const int ts = a.fold ? cr / a.CP : 0;
        const int c = cr - ts * a.CP;
        const int tapi = a.fold ? tb * a.S + ts : tb;
        if (a.direct && c >= a.C) continue;
        float inv_in = 0.f;
        if (a.direct && a.lw && a.l_in) {
            const float in = a.l_in[c];
            inv_in = in > 0.f ? 1.0f / in : 0.f;
        }
        if (a.direct && a.lw) {  // uniform: regulariser folded in
            // every weight and norm this lane needs is fetched before the first store: the stores may alias the loads
            // as far as the compiler knows, and interleaved they would each wait out a full memory round trip
            float wv[TN][16], io[TN][16];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int k = n0 + wn * WTN + tn * 32 + 8 * (e >> 2) + hi4 + (e & 3);
                    const int kc = k < a.K ? k : a.K - 1;
                    wv[tn][e] = a.lw[((int64_t)kc * a.RS + tapi) * a.wpitch + c];
                    io[tn][e] = a.l_on ? a.l_on[kc] : 0.f;
                }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int k = n0 + wn * WTN + tn * 32 + 8 * (e >> 2) + hi4 + (e & 3);
                    if (k >= a.K) continue;
                    const float inv_out = io[tn][e] > 0.f ? 1.0f / io[tn][e] : 0.f;
                    out[((int64_t)k * a.RS + tapi) * a.wpitch + c] =
                        acc[tm][tn][e] + a.l_lambda * (wv[tn][e] * (inv_out + inv_in));
                }
            continue;
        }
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int k = n0 + wn * WTN + tn * 32 + 8 * g + hi4 + i;
                    if (k >= a.K) continue;
                    const float v = acc[tm][tn][4 * g + i];
                    if (a.direct)
                        out[((int64_t)k * a.RS + tapi) * a.wpitch + c] = v;
                    else
                        out[(int64_t)k * a.out_row_pitch + tapi * a.CP + c] = v;
                }
            }
        }
    }
#endif
}

template <int BM, int BN, int BKP, int WGM, int WGN, int STAGES, int KSPLIT, int MINB, int XMODE>
inline hipError_t launch_wgrad_dl_mode(WgradArgs& a, hipStream_t st) {
    constexpr int NT = 64 * WGM * WGN * KSPLIT;
    constexpr size_t ring = (size_t)STAGES * BKP * (BM + BN) * 2, red = KSPLIT > 1 ? (size_t)BM * BN * 4 : 0;
    constexpr size_t lds = ring > red ? ring : red;
    static_assert(lds <= 160 * 1024, "LDS capacity");
    auto kern = k_wgrad_dl<BM, BN, BKP, WGM, WGN, STAGES, KSPLIT, MINB, XMODE>;
    const int P = (int)a.P.d, Q = (int)a.Q.d;
    a.dq = BKP % Q;
    a.dp = (BKP / Q) % P;
    a.dn = BKP / (P * Q);
    static LdsOptIn opt_in;
    if (hipError_t e = opt_in.ensure(reinterpret_cast<const void*>(kern), lds); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(a.tiles_m * a.tiles_n * a.splits), dim3(NT), lds, st, a);
    return hipSuccess;
}

template <int BM, int BN, int BKP, int WGM, int WGN, int STAGES, int KSPLIT = 1, int MINB = 1>
inline hipError_t launch_wgrad_dl_cfg(WgradArgs& a, hipStream_t st) {
    if (a.x_all_valid) return launch_wgrad_dl_mode<BM, BN, BKP, WGM, WGN, STAGES, KSPLIT, MINB, 2>(a, st);
    if (a.affine) return launch_wgrad_dl_mode<BM, BN, BKP, WGM, WGN, STAGES, KSPLIT, MINB, 1>(a, st);
    return launch_wgrad_dl_mode<BM, BN, BKP, WGM, WGN, STAGES, KSPLIT, MINB, 0>(a, st);
}

// ------------------------------------------------------------------------------------------- //
// 3 x 3 convolution at stride 1, padding 1, with at most 64 channels on either side: weights resident in LDS
// ------------------------------------------------------------------------------------------- //
// The early 3 x 3 layers of a network (many pixels, few channels) have nine reduction steps per tile in the
// implicit-GEMM kernel, and a workgroup there spends as long on its set-up, its first loads and its stores as on the
// steps.  Here ONE workgroup per CU keeps the whole filter bank in LDS ([64 outputs][9 taps][64 channels] bf16, rows
// padded by 16 bytes so that the 32 rows a fragment read touches spread over all banks) and walks over a run of tiles of
// 4 x 8*nb output pixels (nb <= 7 column blocks of 8).  Per tile the input patch with its halo, 6 x (8*nb + 2) pixels x
// 128 bytes, goes to one of two LDS buffers by 16-byte global->LDS loads (out-of-image pixels and channels past the
// count fetch zeros), the next tile's patch while the current one is multiplied.  Wave b of the eight owns column block
// b: 4 x 8 pixels x 64 outputs, two accumulator blocks; per (tap, 16 channels) one 16-byte patch read and two weight
// reads feed two MFMAs.  The nine taps are nine windows of the same patch: nothing is fetched twice.  The 16-byte
// chunks of a patch pixel are XOR-ed with ((column >> 1) & 3) | ((row & 1) << 2): the 16 lanes one LDS cycle serves
// (two rows of eight pixels) then read 16 different bank groups, for every tap.  FLIP: the weights are indexed by the
// mirrored tap (input gradient: the same kernel on dy with the k-innermost filter copy).
struct Res3Args {
    const uint16_t* X;   // [N][H][W][ip]
    const uint16_t* Wt;  // [Mout][9][wp], reduction channel innermost
    uint16_t* Y;         // [N][H][W][op]
    int N, H, W, Cin, CinP, ip, Mout, wp, op;  // CinP = Cin rounded up to 8
    int nb;                                  // column blocks of 8 pixels per tile
    int tiles_x, tiles_y, tiles, run;
};
constexpr int kR3TH = 4, kR3MaxNB = 7, kR3PH = kR3TH + 2, kR3PW = 8 * kR3MaxNB + 2;
constexpr int kR3WRow = 9 * 128 + 16, kR3WBytes = 64 * kR3WRow;
constexpr int kR3PatchSlots = kR3PH * kR3PW * 8, kR3PatchBytes = kR3PatchSlots * 16;
constexpr int kR3Lds = kR3WBytes + 2 * kR3PatchBytes;
constexpr int kR3Slots = 256;  // one workgroup per CU
static_assert(kR3Lds <= 160 * 1024 && (64 * (kR3WRow / 16)) % 64 == 0, "LDS plan");

// NCB: 16-channel steps per tap (CinP / 16 rounded up); KB1: more than 32 outputs (the second accumulator block is live).
// Compile-time so that the 9 * NCB steps of a tile are one straight line of code: with a branch per step every fragment
// read is waited out before its MFMA (27 us against 34 us for the implicit-GEMM kernel on 56 x 56 x 64 -> 64;
// straight-line with the reads of step s + 1 issued before the MFMAs of step s: see the numbers in the notes).
template <bool FLIP, int NCB, bool KB1>
__global__ __launch_bounds__(512) void k_conv3x3_res(const Res3Args a) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr uint32_t kBufOut = 0xffffffffu, kBufFlags = 0x00020000u;
    constexpr int WSLOTS = kR3WRow / 16;                       // 16-byte slots per weight row (73, the last one padding)
    constexpr int NWL = 64 * WSLOTS / 64, WL = (NWL + 7) / 8;  // wave-level loads of the weights, per wave
    constexpr int NPL = (kR3PatchSlots + 63) / 64, PL = (NPL + 7) / 8;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_b[];
    uint8_t* wl = smem_b;
    uint8_t* pbuf = smem_b + kR3WBytes;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int first = blockIdx.x * a.run, last = first + a.run < a.tiles ? first + a.run : a.tiles;
    if (first >= last) return;  // whole workgroup

    // ---- filter bank -> LDS, once ---------------------------------------------------------------------------------
    {
        const __amdgpu_buffer_rsrc_t w_srd = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(a.Wt), 0, (uint32_t)(a.Mout * 9 * a.wp) * 2u, kBufFlags);
#pragma unroll
        for (int i = 0; i < WL; ++i) {
            const int idx = wave + 8 * i < NWL ? wave + 8 * i : NWL - 1;  // (past the end: the last one again)
            const int sl = idx * 64 + lane;
            const int m = sl / WSLOTS, wi = sl - m * WSLOTS;
            const int t = wi >> 3, j = wi & 7;
            const bool ok = wi < 72 && m < a.Mout && j * 8 < a.CinP;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(w_srd, (lds_void_ptr)(wl + idx * 1024), 16,
                                                     ok ? (uint32_t)(((m * 9 + t) * a.wp + j * 8) * 2) : kBufOut, 0, 0, 0);
        }
    }
    // ---- this lane's slots of a patch: the same places in every tile ---------------------------------------------------
    int p_rc[PL];        // row << 16 | column, or -1
    uint32_t p_rel[PL];  // byte offset of the chunk from the patch's first pixel
    int p_idx[PL];
#pragma unroll
    for (int i = 0; i < PL; ++i) {
        p_idx[i] = wave + 8 * i < NPL ? wave + 8 * i : NPL - 1;
        const int sl = p_idx[i] * 64 + lane;
        const int pr = sl / (kR3PW * 8), rem = sl - pr * (kR3PW * 8);
        const int pc = rem >> 3, pj = rem & 7;
        const int j = pj ^ (((pc >> 1) & 3) | ((pr & 1) << 2));  // the logical chunk that belongs at this place
        const bool ok = sl < kR3PatchSlots && j * 8 < a.CinP && pc < 8 * a.nb + 2;
        p_rc[i] = ok ? (pr << 16) | pc : (sl < kR3PatchSlots ? -1 : -2);
        p_rel[i] = (uint32_t)(((pr * a.W + pc) * a.ip + j * 8) * 2);
    }
    const uint32_t in_bytes = (uint32_t)(a.H * a.W * a.ip) * 2u, out_bytes = (uint32_t)(a.H * a.W * a.op) * 2u;
    auto decode = [&](int tile, int& tx, int& ty, int& img) {
        tx = tile % a.tiles_x;
        ty = (tile / a.tiles_x) % a.tiles_y;
        img = tile / (a.tiles_x * a.tiles_y);
    };
    auto issue = [&](int tile, int buf) {
        int tx, ty, img;
        decode(tile, tx, ty, img);
        const int ih0 = ty * kR3TH - 1, iw0 = tx * 8 * a.nb - 1;
        const __amdgpu_buffer_rsrc_t x_srd = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(a.X) + (int64_t)img * a.H * a.W * a.ip, 0, in_bytes, kBufFlags);
        const uint32_t xs = (uint32_t)((ih0 * a.W + iw0) * a.ip * 2);
        uint8_t* dst = pbuf + buf * kR3PatchBytes;
#pragma unroll
        for (int i = 0; i < PL; ++i) {
            const int ih = ih0 + (p_rc[i] >> 16), iw = iw0 + (p_rc[i] & 0xffff);
            const bool ok = p_rc[i] >= 0 && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            // (slots past the buffer's end belong to lanes of the last load that must not write at all)
            if (p_rc[i] != -2)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(x_srd, (lds_void_ptr)(dst + p_idx[i] * 1024), 16,
                                                         ok ? p_rel[i] + xs : kBufOut, 0, 0, 0);
        }
    };

    // ---- MFMA state -----------------------------------------------------------------------------------------------
    const int l32 = lane & 31, h = lane >> 5;
    const int pr0 = l32 >> 3, pc0 = wave * 8 + (l32 & 7);  // this lane's output pixel inside the tile
    const bool active = wave < a.nb;
    uint32_t pb[9], pk[9];  // per tap: byte offset of the pixel under it in a patch, and its chunk swizzle (<< 4)
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const int pr = pr0 + t / 3, pc = pc0 + t % 3;
        pb[t] = (uint32_t)((pr * kR3PW + pc) * 128);
        pk[t] = (uint32_t)((((pc >> 1) & 3) | ((pr & 1) << 2)) << 4);
    }
    const uint8_t* wa = wl + l32 * kR3WRow + h * 16;
    const uint32_t hc = (uint32_t)(h << 4);

    issue(first, 0);
    int buf = 0;
    for (int tile = first; tile < last; ++tile, buf ^= 1) {
        const bool more = tile + 1 < last;  // uniform
        // the patch of this tile (and at first the weights) has landed; this wave's stores of the previous tile, which
        // were issued after those loads, may still be in flight (every active wave issues exactly four)
        if (active && tile != first) wait_vmcnt<4>();
        else wait_vmcnt<0>();
        barrier_nofence();
        if (more) issue(tile + 1, buf ^ 1);
        // the loads stay here, ahead of the multiply and of the stores: the wait at the top of the next tile counts on
        // the stores being the last four memory instructions of the wave, and the loads need the multiply's time to land
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        if (active) {
            int tx, ty, img;
            decode(tile, tx, ty, img);
            f32x16 acc[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[kb][v] = 0.f;
            const uint8_t* pp = pbuf + buf * kR3PatchBytes;
            bf16x8 xb[2], w0[2], w1[2];
            auto read_frags = [&](auto s_c) {
                constexpr int S = decltype(s_c)::value, t = S / NCB, cb = S % NCB, B = S & 1, tw = FLIP ? 8 - t : t;
                xb[B] = *reinterpret_cast<const bf16x8*>(pp + pb[t] + (((uint32_t)(cb << 5) | hc) ^ pk[t]));
                w0[B] = *reinterpret_cast<const bf16x8*>(wa + tw * 128 + cb * 32);
                if constexpr (KB1) w1[B] = *reinterpret_cast<const bf16x8*>(wa + 32 * kR3WRow + tw * 128 + cb * 32);
            };
            read_frags(std::integral_constant<int, 0>{});
            static_for<0, 9 * NCB>([&](auto s_c) {
                constexpr int S = decltype(s_c)::value, B = S & 1;
                if constexpr (S + 1 < 9 * NCB) read_frags(std::integral_constant<int, S + 1>{});
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w0[B], xb[B], acc[0], 0, 0, 0);
                if constexpr (KB1) acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1[B], xb[B], acc[1], 0, 0, 0);
            });
            // ---- store: the lane-pair exchange of k_igemm_dl (64 contiguous bytes per pixel pair and output block) -----
            const __amdgpu_buffer_rsrc_t y_srd = __builtin_amdgcn_make_buffer_rsrc(
                a.Y + (int64_t)img * a.H * a.W * a.op, 0, out_bytes, kBufFlags);
            const int oh = ty * kR3TH + pr0, ow = tx * 8 * a.nb + pc0;
            const bool odd = (lane & 1) != 0;
            const int chl = (odd ? 16 : 0) + 8 * h;
            const bool row_ok = oh < a.H;
            const bool ok0 = row_ok && (ow & ~1) < a.W, ok1 = row_ok && (ow | 1) < a.W;
            const uint32_t pix0 = (uint32_t)((oh * a.W + (ow & ~1)) * a.op) * 2u;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const int ch = kb * 32 + chl;
                const f32x16& c = acc[kb];
                uint32_t v[2][4];
#pragma unroll
                for (int gp = 0; gp < 2; ++gp) {
                    const uint32_t x0 = cvt_pk_bf16(c[8 * gp + 0], c[8 * gp + 1]), y0 = cvt_pk_bf16(c[8 * gp + 2], c[8 * gp + 3]);
                    const uint32_t x1 = cvt_pk_bf16(c[8 * gp + 4], c[8 * gp + 5]), y1 = cvt_pk_bf16(c[8 * gp + 6], c[8 * gp + 7]);
                    const auto ps = __builtin_amdgcn_permlane32_swap(x0, x1, false, false);
                    const auto qs = __builtin_amdgcn_permlane32_swap(y0, y1, false, false);
                    v[gp][0] = ps[0]; v[gp][1] = qs[0]; v[gp][2] = ps[1]; v[gp][3] = qs[1];
                }
                uint32_t s0[4], s1[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t give = odd ? v[0][e] : v[1][e];
                    const uint32_t got = (uint32_t)__shfl_xor((int)give, 1, 64);
                    s0[e] = odd ? got : v[0][e];
                    s1[e] = odd ? v[1][e] : got;
                }
                uint4 o0 = make_uint4(s0[0], s0[1], s0[2], s0[3]), o1 = make_uint4(s1[0], s1[1], s1[2], s1[3]);
                const bool ch_ok = ch < a.Mout;
                if (ch_ok && ch + 7 >= a.Mout) {  // last chunk: zeros in its padding
                    const Mask8 k = make_mask8(a.Mout - ch);
                    o0 = mask8(o0, true, k);
                    o1 = mask8(o1, true, k);
                }
                const uint32_t off0 = pix0 + (uint32_t)ch * 2u;
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o0), y_srd, ok0 && ch_ok ? off0 : kBufOut, 0, 0);
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o1), y_srd,
                                                       ok1 && ch_ok ? off0 + (uint32_t)a.op * 2u : kBufOut, 0, 0);
            }
        }
    }
#endif
}

inline hipError_t launch_conv3x3_res(Res3Args& a, bool flip, hipStream_t st) {
    const int nbw = (a.W + 7) / 8;
    a.nb = nbw < kR3MaxNB ? nbw : kR3MaxNB;
    a.tiles_x = (a.W + 8 * a.nb - 1) / (8 * a.nb);
    a.tiles_y = (a.H + kR3TH - 1) / kR3TH;
    const int64_t tiles = (int64_t)a.N * a.tiles_x * a.tiles_y;
    if (tiles <= 0 || tiles > 0x3fffffff) return hipErrorInvalidValue;
    a.tiles = (int)tiles;
    a.run = (int)((tiles + kR3Slots - 1) / kR3Slots);
    const unsigned grid = (unsigned)((tiles + a.run - 1) / a.run);
    typedef void (*kern_t)(const Res3Args);
    static const kern_t kerns[2][4][2] = {
        {{k_conv3x3_res<false, 1, false>, k_conv3x3_res<false, 1, true>}, {k_conv3x3_res<false, 2, false>, k_conv3x3_res<false, 2, true>},
         {k_conv3x3_res<false, 3, false>, k_conv3x3_res<false, 3, true>}, {k_conv3x3_res<false, 4, false>, k_conv3x3_res<false, 4, true>}},
        {{k_conv3x3_res<true, 1, false>, k_conv3x3_res<true, 1, true>}, {k_conv3x3_res<true, 2, false>, k_conv3x3_res<true, 2, true>},
         {k_conv3x3_res<true, 3, false>, k_conv3x3_res<true, 3, true>}, {k_conv3x3_res<true, 4, false>, k_conv3x3_res<true, 4, true>}}};
    static LdsOptIn opt_in[2][4][2];
    const int ncb = (a.CinP + 15) / 16, kb1 = a.Mout > 32 ? 1 : 0;
    if (ncb < 1 || ncb > 4) return hipErrorInvalidValue;
    const kern_t kern = kerns[flip ? 1 : 0][ncb - 1][kb1];
    if (hipError_t e = opt_in[flip ? 1 : 0][ncb - 1][kb1].ensure(reinterpret_cast<const void*>(kern), kR3Lds); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), kR3Lds, st, a);
    return hipSuccess;
}

// ------------------------------------------------------------------------------------------- //
// weight gradient of a network's first layer: image-like input, at most 4 channels at a pitch of 8
// ------------------------------------------------------------------------------------------- //
// dw[k][r][s][c] = sum over output pixels of dy[pixel][k] * x[pixel * stride + (r, s)][c] (Eq. 4).  As in k_stem_fwd
// the unit of work is a tile of output pixels (2 x 64) whose input patch is loaded once; here the dy tile comes along
// and both go to LDS by 16-byte global->LDS loads: dy rows of 64 channels = 128 bytes with the unit swizzle of
// k_wgrad_dl's 128-byte rows, the patch in image order at 16 bytes per pixel (the 4 padding channels ride along).
// The reduction runs over the tile's pixels, 16 per MFMA step: wave r of a group of eight owns filter row r and
// accumulates 64 output channels (two 32 x 32 blocks) x 32 columns = 8 taps x 4 channels.  Both fragments are
// transposing reads: of dy as in k_wgrad_dl; of the patch, a source lane points at the 4 channels of pixel
// (q + row) * stride + tap, so the 16 columns of a read are 4 taps x 4 channels and its rows 4 consecutive output
// pixels.  A workgroup has two such groups of eight waves working on alternate tiles of one run of tiles, each with
// its own double-buffered LDS region; at the end the second group's sums are added to the first's through LDS and ONE
// slab of fp32 partial sums per workgroup, [r][64][32], goes to the workspace.  One workgroup per CU: the slabs of a
// launch are 256 x 57 KB, summed in a fixed order by k_stem_wgrad_reduce (which also adds the regulariser's term).
struct StemWgradArgs {
    const uint16_t* X;   // [N][H][W][8]
    const uint16_t* DY;  // [N][P][Q][ypitch]
    float* PART;         // [workgroup][R][64][32]
    int N, H, W, P, Q, K, KP, R, S, pad_h, pad_w, ypitch;
    int tiles_q, tiles_p;  // tiles per image along Q and P
    int tiles, run;        // N * tiles_p * tiles_q, and how many consecutive tiles one workgroup takes
};
constexpr int kSwTH = 2, kSwTW = 64;
constexpr int kSwSlots = 256;                 // one workgroup of 16 waves per CU
constexpr int kSwSlabRow = 64 * 32;           // floats per filter row in a slab

template <int STRIDE>
__global__ __launch_bounds__(1024) void k_stem_wgrad(const StemWgradArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int PH = (kSwTH - 1) * STRIDE + kStemMaxR;   // patch rows (for the largest filter)
    constexpr int PW = (kSwTW - 1) * STRIDE + 8;           // patch columns: 8 taps per filter row
    constexpr int NXL = (PH * PW + 63) / 64;               // wave-level loads of a patch, 64 pixels each
    constexpr int XL = (NXL + 7) / 8;                      // per wave
    constexpr int YL = kSwTH * kSwTW / 8 / 8;              // dy: 8 pixels per wave-level load, 8 waves
    constexpr int YB = kSwTH * kSwTW * 128, XB = NXL * 1024, STAGE = YB + XB, GROUP = 2 * STAGE;
    constexpr uint32_t kBufOut = 0xffffffffu, kBufFlags = 0x00020000u;
    static_assert(YL == 2 && 2 * GROUP <= 160 * 1024, "tile config");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_b[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hh = wave >> 3, w8 = wave & 7;     // group of eight waves, wave inside it = filter row
    const int first = blockIdx.x * a.run, last = first + a.run < a.tiles ? first + a.run : a.tiles;
    const int niter = (a.run + 1) >> 1;          // the same for every workgroup: tiles past `last` are fetched as zeros
    const bool active = w8 < a.R;
    const int ph_used = (kSwTH - 1) * STRIDE + a.R;
    uint8_t* gbase = smem_b + hh * GROUP;

    // ---- loader state ---------------------------------------------------------------------------------------------
    // dy: wave-level load d = w8 + 8 i covers pixels 8 d .. 8 d + 7 of the tile (i = tile row), a lane one 16-byte chunk;
    // the chunk a lane fetches is the logical one that belongs at its physical place in the swizzled row
    const int yq = 8 * w8 + (lane >> 3);         // output column inside the tile
    uint32_t y_v[YL];
    {
        const int pc = lane & 7, sw = (yq >> 1) & 1;         // (the pixel row's swizzle bit: rows i * 64 + yq)
        const int qq = (pc >> 1) ^ sw;
        const int lc = ((((qq & 1) << 1) | (qq >> 1)) << 1) | (pc & 1);
#pragma unroll
        for (int i = 0; i < YL; ++i) y_v[i] = lc * 8 < a.KP ? (uint32_t)(((i * a.Q + yq) * a.ypitch + lc * 8) * 2) : kBufOut;
    }
    // patch: wave-level load idx covers pixels 64 idx .. 64 idx + 63 of the patch in row-major order; loads past the
    // last one repeat it (same data to the same place), so that every wave issues the same number
    int x_rc[XL];          // row << 16 | column, or -1
    uint32_t x_rel[XL];    // byte offset of the pixel from the patch's first pixel
    int x_idx[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) {
        x_idx[i] = w8 + 8 * i < NXL ? w8 + 8 * i : NXL - 1;
        const int slot = x_idx[i] * 64 + lane;
        const int prow = slot / PW, pcol = slot - prow * PW;
        x_rc[i] = prow < ph_used && prow < PH ? (prow << 16) | pcol : -1;
        x_rel[i] = (uint32_t)(prow * a.W + pcol) * 16u;
    }
    const uint32_t img_bytes = (uint32_t)(a.H * a.W) * 16u;

    auto issue = [&](int tile, int stage) {
        const bool tv = tile < last;  // uniform
        const int tq = tile % a.tiles_q;
        const int tp = (tile / a.tiles_q) % a.tiles_p;
        const int img = tile / (a.tiles_q * a.tiles_p);
        const int p0 = tp * kSwTH, q0 = tq * kSwTW;
        uint8_t* sbase = gbase + stage * STAGE;
        const __amdgpu_buffer_rsrc_t y_srd = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(a.DY) + ((int64_t)(img * a.P + p0) * a.Q + q0) * a.ypitch, 0, 0xffffff00u, kBufFlags);
        const bool q_ok = tv && q0 + yq < a.Q;
#pragma unroll
        for (int i = 0; i < YL; ++i) {
            const uint32_t v = q_ok && p0 + i < a.P ? y_v[i] : kBufOut;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(y_srd, (lds_void_ptr)(sbase + (w8 + 8 * i) * 1024), 16, v, 0, 0, 0);
        }
        const __amdgpu_buffer_rsrc_t x_srd = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(a.X) + (int64_t)img * a.H * a.W * 8, 0, img_bytes, kBufFlags);
        const int ih0 = p0 * STRIDE - a.pad_h, iw0 = q0 * STRIDE - a.pad_w;
        const uint32_t xs = (uint32_t)((ih0 * a.W + iw0) * 16);
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int ih = ih0 + (x_rc[i] >> 16), iw = iw0 + (x_rc[i] & 0xffff);
            const bool ok = tv && x_rc[i] >= 0 && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(x_srd, (lds_void_ptr)(sbase + YB + x_idx[i] * 1024), 16,
                                                     ok ? x_rel[i] + xs : kBufOut, 0, 0, 0);
        }
    };

    // ---- MFMA state -----------------------------------------------------------------------------------------------
    // transpose-read geometry: 16-lane group g16, lane t16; source lane t16 points at pixel row (t16 >> 2) and 8-byte
    // quad (t16 & 3); the result is 4 consecutive pixels for column 16 * (g16 & 1) + t16
    const int g16 = lane >> 4, t16 = lane & 15;
    const int tr_row = (g16 >> 1) * 8 + (t16 >> 2);   // + 4 h + 16 (step inside the tile row)
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void_ptr)gbase;
    uint32_t ay[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        const int u = 2 * kb + (g16 & 1);              // 32-byte unit (16 channels) of the 128-byte row
        const int up = (((u & 1) << 1) | (u >> 1)) ^ ((tr_row >> 1) & 1);
        ay[kb] = lds0 + (uint32_t)(tr_row * 128 + (up << 5) + (t16 & 3) * 8);
    }
    // patch: filter row w8, pixel (tile column tr_row) * STRIDE + tap, tap = 4 (g16 & 1) + (t16 & 3)
    const uint32_t ax = lds0 + (uint32_t)(YB + (w8 * PW + tr_row * STRIDE + 4 * (g16 & 1) + (t16 & 3)) * 16);
    f32x16 acc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[kb][v] = 0.f;

    // One tile: 8 steps of 16 pixels (tile row pl = step / 4); the reads of step st + 1 are in flight during the MFMAs of st.
    auto compute = [&](int stage) {
        const uint32_t sb = (uint32_t)(stage * STAGE);
        const uint32_t by0 = ay[0] + sb, by1 = ay[1] + sb, bx = ax + sb;
        s16x4 fy[2][2][2], fx[2][2];
        auto issue_reads = [&](auto st_c) {
            constexpr int ST = decltype(st_c)::value, PL = ST >> 2, KQ = ST & 3, B = ST & 1;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (h == 0) {
                    fy[B][0][0] = lds_read_tr16_b64<(PL * 64 + 16 * KQ) * 128>(by0);
                    fy[B][1][0] = lds_read_tr16_b64<(PL * 64 + 16 * KQ) * 128>(by1);
                    fx[B][0] = lds_read_tr16_b64<(PL * STRIDE * PW + 16 * KQ * STRIDE) * 16>(bx);
                } else {
                    fy[B][0][1] = lds_read_tr16_b64<(PL * 64 + 16 * KQ + 4) * 128>(by0);
                    fy[B][1][1] = lds_read_tr16_b64<(PL * 64 + 16 * KQ + 4) * 128>(by1);
                    fx[B][1] = lds_read_tr16_b64<(PL * STRIDE * PW + (16 * KQ + 4) * STRIDE) * 16>(bx);
                }
            }
        };
        issue_reads(std::integral_constant<int, 0>{});
        static_for<0, 8>([&](auto st_c) {
            constexpr int ST = decltype(st_c)::value, B = ST & 1;
            if constexpr (ST + 1 < 8) {
                issue_reads(std::integral_constant<int, ST + 1>{});
                lds_wait<6>(fy[B][0][0]);
            } else {
                lds_wait<0>(fy[B][0][0]);
            }
            lds_tie(fy[B][0][1]); lds_tie(fy[B][1][0]); lds_tie(fy[B][1][1]); lds_tie(fx[B][0]); lds_tie(fx[B][1]);
            const bf16x8 vx = join_halves(fx[B][0], fx[B][1]);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
                acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(join_halves(fy[B][kb][0], fy[B][kb][1]), vx, acc[kb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // ---- tiles first + hh, first + hh + 2, ...: loads one tile ahead, one barrier per tile ------------------------------
    issue(first + hh, 0);
    for (int it = 0; it < niter; ++it) {
        wait_vmcnt<0>();      // this wave's loads of tile `it` have landed ...
        barrier_nofence();    // ... and everybody's; everybody is also done reading the other stage
        if (it + 1 < niter) issue(first + hh + 2 * (it + 1), (it + 1) & 1);
        if (active) compute(it & 1);
    }

    // ---- the second group's sums join the first's through LDS; one slab per workgroup ---------------------------------
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem_b);
    if (hh == 1 && active) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) red[((w8 * 2 + kb) * 16 + v) * 64 + lane] = acc[kb][v];
    }
    __syncthreads();
    if (hh == 0 && active) {
        const int l32 = lane & 31, h = lane >> 5;
        float* slab = a.PART + ((int64_t)blockIdx.x * a.R + w8) * kSwSlabRow;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = kb * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                slab[k * 32 + l32] = acc[kb][v] + red[((w8 * 2 + kb) * 16 + v) * 64 + lane];
            }
    }
#endif
}

inline size_t stem_wgrad_lds(int stride) {
    const int ph = (kSwTH - 1) * stride + kStemMaxR, pw = (kSwTW - 1) * stride + 8;
    return (size_t)4 * (kSwTH * kSwTW * 128 + (ph * pw + 63) / 64 * 1024);
}

// Fills in the tiling; `slabs` = workgroups of the launch = slabs of partial sums written.
inline void plan_stem_wgrad(StemWgradArgs& a, int* slabs) {
    a.tiles_q = (a.Q + kSwTW - 1) / kSwTW;
    a.tiles_p = (a.P + kSwTH - 1) / kSwTH;
    const int64_t tiles = (int64_t)a.N * a.tiles_p * a.tiles_q;
    a.tiles = (int)tiles;
    a.run = (int)((tiles + kSwSlots - 1) / kSwSlots);
    if (a.run < 1) a.run = 1;
    *slabs = (int)((tiles + a.run - 1) / a.run);
}

inline hipError_t launch_stem_wgrad(const StemWgradArgs& a, int slabs, int stride, hipStream_t st) {
    const size_t lds = stem_wgrad_lds(stride);
    static LdsOptIn opt_in[2];
    if (stride == 1) {
        if (hipError_t e = opt_in[0].ensure(reinterpret_cast<const void*>(k_stem_wgrad<1>), lds); e != hipSuccess) return e;
        hipLaunchKernelGGL(k_stem_wgrad<1>, dim3((unsigned)slabs), dim3(1024), lds, st, a);
    } else {
        if (hipError_t e = opt_in[1].ensure(reinterpret_cast<const void*>(k_stem_wgrad<2>), lds); e != hipSuccess) return e;
        hipLaunchKernelGGL(k_stem_wgrad<2>, dim3((unsigned)slabs), dim3(1024), lds, st, a);
    }
    return hipSuccess;
}

}  // namespace pt
