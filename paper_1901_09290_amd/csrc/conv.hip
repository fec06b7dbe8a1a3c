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
#include "common.h"

namespace pt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int kConvThreads = 256;

// 8 bf16 from p; elements [nvalid, 8) are returned as zero.  vec: p is 16-byte aligned and the
// whole 16 bytes are readable.
__device__ __forceinline__ uint4 load8(const uint16_t* __restrict__ p, int nvalid, bool vec) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (nvalid <= 0) return v;
    if (vec) {
        v = *reinterpret_cast<const uint4*>(p);
        if (nvalid < 8) {
            uint32_t* d = reinterpret_cast<uint32_t*>(&v);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (nvalid <= 2 * i) d[i] = 0u;
                else if (nvalid == 2 * i + 1) d[i] &= 0xffffu;
            }
        }
    } else {
        uint32_t* d = reinterpret_cast<uint32_t*>(&v);
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (e < nvalid) d[e >> 1] |= (uint32_t)p[e] << ((e & 1) * 16);
    }
    return v;
}

// ------------------------------------------------------------------------------------------- //
// forward / input-gradient implicit GEMM
// ------------------------------------------------------------------------------------------- //
struct IgemmArgs {
    const uint16_t* A;  // gathered activations (x or dy)
    const uint16_t* B;  // weights, [Nout][b_taps][bpitch], reduction channel innermost
    uint16_t* D;        // output activations
    int M;              // output pixels of this launch = images * gH * gW
    int gH, gW;         // output pixel grid per image (of this launch)
    int srcH, srcW, apitch;
    int h_mul, h_add, w_mul, w_add;  // source coordinate of tap (0,0) for grid point (i,j)
    int tr_step, ts_step;            // source coordinate step per tap index
    int TR, TS;                      // taps of this launch
    int Cred, CredP;                 // reduction channels, and rounded up to 8
    int b_tap0, b_tr_stride, b_ts_stride, b_taps;
    int bpitch, Nout;
    int DH, DW, d_hmul, d_hadd, d_wmul, d_wadd, dpitch;  // destination pixel = (i*d_hmul+d_hadd, j*d_wmul+d_wadd)
    int nk;                                              // reduction steps of BK
    int tiles_n;
    int a_vec, b_vec, d_vec;
};

// XCD-aware block remap: hardware deals consecutive workgroup ids round-robin to the 8 XCDs; give
// each XCD a contiguous range of logical tiles so tiles that share operands share an L2.
__device__ __forceinline__ int xcd_remap(int bid, int nb) {
    const int xcd = bid & 7, q = bid >> 3;
    const int per = nb >> 3, rem = nb & 7;
    return xcd * per + min(xcd, rem) + q;
}

template <int BM, int BN, int BK, int WGM, int WGN>
__global__ __launch_bounds__(kConvThreads) void k_igemm(const IgemmArgs a) {
    constexpr int LDK = BK + 8;  // LDS row pitch in elements (16-byte pad: conflict-free 16-byte reads)
    constexpr int KV = BK / 8;
    constexpr int RPP = kConvThreads / KV;
    constexpr int AP = BM / RPP, BP = BN / RPP;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert(WGM * WGN == 4 && AP >= 1 && BP >= 1 && TM >= 1 && TN >= 1, "tile config");
    __shared__ __attribute__((aligned(16))) uint16_t sA[2][BM * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t sB[2][BN * LDK];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    int a_h0[AP], a_w0[AP];
    int64_t a_base[AP];
    const int gHW = a.gH * a.gW;
#pragma unroll
    for (int i = 0; i < AP; ++i) {
        const int m = m0 + lrow + i * RPP;
        if (m < a.M) {
            const int n = m / gHW, rem = m - n * gHW;
            const int gi = rem / a.gW, gj = rem - gi * a.gW;
            a_h0[i] = gi * a.h_mul + a.h_add;
            a_w0[i] = gj * a.w_mul + a.w_add;
            a_base[i] = (int64_t)n * a.srcH * a.srcW;
        } else {
            a_h0[i] = -(1 << 28);  // never in bounds
            a_w0[i] = 0;
            a_base[i] = 0;
        }
    }
    int64_t b_base[BP];
    bool b_ok[BP];
#pragma unroll
    for (int j = 0; j < BP; ++j) {
        const int nrow = n0 + lrow + j * RPP;
        b_ok[j] = nrow < a.Nout;
        b_base[j] = (int64_t)nrow * a.b_taps * a.bpitch;
    }

    uint4 ra[AP], rb[BP];
    auto gload = [&]() {
        const bool kok = tr < a.TR;
        const int nvalid = kok ? a.Cred - c0 : 0;
        const int dh = tr * a.tr_step, dw = ts * a.ts_step;
#pragma unroll
        for (int i = 0; i < AP; ++i) {
            const int ih = a_h0[i] + dh, iw = a_w0[i] + dw;
            const bool ok = (unsigned)ih < (unsigned)a.srcH && (unsigned)iw < (unsigned)a.srcW;
            const int64_t off = (a_base[i] + (int64_t)ih * a.srcW + iw) * a.apitch + c0;
            ra[i] = load8(a.A + (ok ? off : 0), ok ? nvalid : 0, a.a_vec);
        }
        const int tapw = a.b_tap0 + tr * a.b_tr_stride + ts * a.b_ts_stride;
#pragma unroll
        for (int j = 0; j < BP; ++j) {
            const int64_t off = b_base[j] + (int64_t)tapw * a.bpitch + c0;
            rb[j] = load8(a.B + (b_ok[j] && kok ? off : 0), b_ok[j] ? nvalid : 0, a.b_vec);
        }
        // advance to the next reduction step
        c0 += BK;
        while (c0 >= a.CredP && tr < a.TR) {
            c0 -= a.CredP;
            if (++ts == a.TS) { ts = 0; ++tr; }
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < AP; ++i)
            *reinterpret_cast<uint4*>(&sA[buf][(lrow + i * RPP) * LDK + kv * 8]) = ra[i];
#pragma unroll
        for (int j = 0; j < BP; ++j)
            *reinterpret_cast<uint4*>(&sB[buf][(lrow + j * RPP) * LDK + kv * 8]) = rb[j];
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

    gload();
    sstore(0);
    __syncthreads();
    for (int kt = 0; kt < a.nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < a.nk) gload();
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fw[TN], fp[TM];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                fw[tn] = *reinterpret_cast<const bf16x8*>(&sB[buf][(wn * WTN + tn * 32 + l32) * LDK + ks * 16 + lk]);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                fp[tm] = *reinterpret_cast<const bf16x8*>(&sA[buf][(wm * WTM + tm * 32 + l32) * LDK + ks * 16 + lk]);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    if (n_live[tn] && m_live[tm])
                        acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[tn], fp[tm], acc[tn][tm], 0, 0, 0);
        }
        if (kt + 1 < a.nk) sstore(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds pixel (column) l32, channels 8g + 4*(lane/32) + {0..3} of each block --
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int m = m0 + wm * WTM + tm * 32 + l32;
        if (m >= a.M) continue;
        const int n = m / gHW, rem = m - n * gHW;
        const int gi = rem / a.gW, gj = rem - gi * a.gW;
        const int64_t dpix =
            (((int64_t)n * a.DH + gi * a.d_hmul + a.d_hadd) * a.DW + gj * a.d_wmul + a.d_wadd) * a.dpitch;
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

// Zero the destination pixels of a stride-parity class that no output pixel reaches.
__global__ void k_zero_class(uint16_t* __restrict__ D, int64_t pixels, int gH, int gW, int DH, int DW, int d_hmul,
                             int d_hadd, int d_wmul, int d_wadd, int dpitch, int Nout) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= pixels * Nout) return;
    const int64_t m = t / Nout;
    const int ch = (int)(t - m * Nout);
    const int gHW = gH * gW;
    const int64_t n = m / gHW;
    const int rem = (int)(m - n * gHW);
    const int gi = rem / gW, gj = rem - gi * gW;
    D[((n * DH + gi * d_hmul + d_hadd) * DW + gj * d_wmul + d_wadd) * dpitch + ch] = 0;
}

// ------------------------------------------------------------------------------------------- //
// weight gradient
// ------------------------------------------------------------------------------------------- //
struct WgradArgs {
    const uint16_t* X;   // x[N][H][W][xpitch]
    const uint16_t* DY;  // dy[pixels][ypitch]
    float* OUT;          // splits > 1: partial[split][K][Mtot]; else dw[K][RS][wpitch]
    int pixels;          // N*P*Q
    int P, Q, H, W, xpitch, ypitch;
    uint32_t magicQ, magicP;
    int stride_h, stride_w, pad_h, pad_w;
    int S, RS, C, CP;    // CP = C rounded up to 8; Mtot = RS*CP
    int Mtot, K;
    int tiles_n;         // tiles along K
    int iters_total, iters_per_split, splits;
    int out_row_pitch;   // elements between consecutive k in OUT (Mtot, or RS*wpitch when direct)
    int wpitch;
    int direct;          // 1: write dw layout directly (splits == 1)
    int x_vec, y_vec, o_vec;
};

template <int BM, int BN, int BK, int WGM, int WGN>
__global__ __launch_bounds__(kConvThreads) void k_wgrad(const WgradArgs a) {
    // LDS tiles are [pixel][channel] with a row pad of 32 elements (64 bytes): the four pixel rows a
    // 16-lane group touches in one transpose read then fall into different banks.
    constexpr int LDM = BM + 32, LDN = BN + 32;
    constexpr int XV = BM / 8, YV = BN / 8;          // 8-vectors per pixel row
    constexpr int XR = kConvThreads / XV, YR = kConvThreads / YV;  // pixel rows per pass
    constexpr int XP = BK / XR, YP = BK / YR;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert(WGM * WGN == 4 && XP >= 1 && YP >= 1 && TM >= 1 && TN >= 1 && BK % 16 == 0, "tile config");
    __shared__ __attribute__((aligned(16))) uint16_t sX[2][BK * LDM];
    __shared__ __attribute__((aligned(16))) uint16_t sY[2][BK * LDN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int n0 = (tile % a.tiles_n) * BN;   // k origin
    const int m0 = (tile / a.tiles_n) * BM;   // (tap, c) origin
    const int split = blockIdx.y;
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

    uint4 rx[XP], ry[YP];
    auto gload = [&](int it) {
        const int pbase = it * BK;
#pragma unroll
        for (int i = 0; i < XP; ++i) {
            const int pix = pbase + xrow + i * XR;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (pix < a.pixels && x_nvalid > 0) {
                const uint32_t row = a.Q == 1 ? (uint32_t)pix : fast_div((uint32_t)pix, a.magicQ);
                const int q = pix - (int)row * a.Q;
                const uint32_t n = a.P == 1 ? row : fast_div(row, a.magicP);
                const int p = (int)row - (int)n * a.P;
                const int ih = p * a.stride_h - a.pad_h + fr, iw = q * a.stride_w - a.pad_w + fs;
                if ((unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W) {
                    const int64_t off = (((int64_t)n * a.H + ih) * a.W + iw) * a.xpitch + xc0;
                    v = load8(a.X + off, x_nvalid, a.x_vec);
                }
            }
            rx[i] = v;
        }
#pragma unroll
        for (int i = 0; i < YP; ++i) {
            const int pix = pbase + yrow + i * YR;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (pix < a.pixels && y_nvalid > 0) v = load8(a.DY + (int64_t)pix * a.ypitch + yk0, y_nvalid, a.y_vec);
            ry[i] = v;
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XP; ++i)
            *reinterpret_cast<uint4*>(&sX[buf][(xrow + i * XR) * LDM + xcv * 8]) = rx[i];
#pragma unroll
        for (int i = 0; i < YP; ++i)
            *reinterpret_cast<uint4*>(&sY[buf][(yrow + i * YR) * LDN + ycv * 8]) = ry[i];
    };

    // ---- MFMA state ---------------------------------------------------------------------------
    const int wm = wave % WGM, wn = wave / WGM;
    // transpose-read geometry: 16-lane group g, lane t in group; source lane t points at pixel row
    // (t/4) and channel quad (t%4); the result is 4 consecutive pixels for channel 16*(g&1) + t.
    const int g16 = lane >> 4, t16 = lane & 15;
    const int tr_row = (g16 >> 1) * 8 + (t16 >> 2);       // + 4*h + ks*16
    const int tr_col = (g16 & 1) * 16 + (t16 & 3) * 4;    // + block origin
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
    for (int it = it0; it < it1; ++it) {
        const int buf = (it - it0) & 1;
        if (it + 1 < it1) gload(it + 1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fx[TM], fy[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                fx[tm] = tr_read(sX[buf], LDM, ks * 16 + tr_row, wm * WTM + tm * 32 + tr_col);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                fy[tn] = tr_read(sY[buf], LDN, ks * 16 + tr_row, wn * WTN + tn * 32 + tr_col);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    if (m_live[tm] && n_live[tn])
                        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[tm], fy[tn], acc[tm][tn], 0, 0, 0);
        }
        if (it + 1 < it1) sstore(buf ^ 1);
        __syncthreads();
    }

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

// dw[k][tap][c] = sum over splits (ascending) of partial[split][k][tap*CP + c].
__global__ void k_wgrad_reduce(const float* __restrict__ part, int splits, int K, int RS, int C, int CP, int wpitch,
                               float* __restrict__ dw) {
    const int Mtot = RS * CP;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)K * Mtot) return;
    const int64_t k = t / Mtot;
    const int mrow = (int)(t - k * Mtot);
    const int tp = mrow / CP, c = mrow - tp * CP;
    if (c >= C) return;
    float s = 0.f;
    for (int i = 0; i < splits; ++i) s += part[(int64_t)i * K * Mtot + t];
    dw[(k * RS + tp) * wpitch + c] = s;
}

// ------------------------------------------------------------------------------------------- //
// host side
// ------------------------------------------------------------------------------------------- //
static int32_t check_desc(const pt_conv_desc* d) {
    if (!d) return PT_ERR_NULL;
    if (d->struct_size != sizeof(pt_conv_desc)) return PT_ERR_SHAPE;
    if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0) return PT_ERR_SHAPE;
    if (d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0) return PT_ERR_SHAPE;
    if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S) return PT_ERR_SHAPE;
    if (d->P != (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1) return PT_ERR_SHAPE;
    if (d->Q != (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1) return PT_ERR_SHAPE;
    if (d->x_cpitch < d->C || d->y_cpitch < d->K || d->w_cpitch < d->C) return PT_ERR_SHAPE;
    // limits of the 32-bit pixel arithmetic inside the kernels
    const int64_t in_pix = (int64_t)d->N * d->H * d->W, out_pix = (int64_t)d->N * d->P * d->Q;
    if (in_pix >= (1ll << 30) || out_pix >= (1ll << 30)) return PT_ERR_UNSUPPORTED;
    if (out_pix * (d->P > d->Q ? d->P : d->Q) >= (1ll << 32)) return PT_ERR_UNSUPPORTED;
    if ((int64_t)d->R * d->S * round_up(d->C, 8) >= (1ll << 30)) return PT_ERR_UNSUPPORTED;
    if ((int64_t)d->R * d->S * round_up(d->K, 8) >= (1ll << 30)) return PT_ERR_UNSUPPORTED;
    return PT_OK;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

template <int BM, int BN, int BK, int WGM, int WGN>
static void launch_igemm_cfg(IgemmArgs& a, hipStream_t st) {
    const int tiles_m = (int)ceil_div(a.M, BM);
    a.tiles_n = (int)ceil_div(a.Nout, BN);
    a.nk = (int)ceil_div((int64_t)a.TR * a.TS * a.CredP, BK);
    hipLaunchKernelGGL((k_igemm<BM, BN, BK, WGM, WGN>), dim3(tiles_m * a.tiles_n), dim3(kConvThreads), 0, st, a);
}

static void launch_igemm(IgemmArgs& a, hipStream_t st) {
    if (a.Nout <= 64)
        launch_igemm_cfg<256, 64, 32, 4, 1>(a, st);
    else
        launch_igemm_cfg<128, 128, 32, 2, 2>(a, st);
}

static size_t bwd_data_ws(const pt_conv_desc* d) {
    return (size_t)round_up((int64_t)d->C * d->R * d->S * round_up(d->K, 8) * 2, 256);
}

struct WgradPlan {
    int splits, iters_total, iters_per_split, tiles_m, tiles_n, CP, Mtot;
    size_t ws_bytes;
};
constexpr int kWgBM = 128, kWgBN = 128, kWgBK = 32;

static WgradPlan plan_wgrad(const pt_conv_desc* d) {
    WgradPlan p;
    p.CP = (int)round_up(d->C, 8);
    p.Mtot = d->R * d->S * p.CP;
    p.tiles_m = (int)ceil_div(p.Mtot, kWgBM);
    p.tiles_n = (int)ceil_div(d->K, kWgBN);
    const int64_t pixels = (int64_t)d->N * d->P * d->Q;
    p.iters_total = (int)ceil_div(pixels, kWgBK);
    const int tiles = p.tiles_m * p.tiles_n;
    int64_t splits = ceil_div(1024, tiles);
    const int64_t max_splits = p.iters_total / 8 > 0 ? p.iters_total / 8 : 1;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    p.iters_per_split = (int)ceil_div(p.iters_total, splits);
    p.splits = (int)ceil_div(p.iters_total, p.iters_per_split);
    p.ws_bytes = p.splits > 1 ? (size_t)round_up((int64_t)p.splits * d->K * p.Mtot * 4, 256) : 0;
    return p;
}

}  // namespace pt

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
    *bytes = plan_wgrad(d).ws_bytes;
    return PT_OK;
}

extern "C" int32_t pt_conv_fwd(const pt_conv_desc* d, const uint16_t* x, const uint16_t* w, uint16_t* y, void* ws,
                               size_t ws_bytes, void* stream) {
    (void)ws;
    (void)ws_bytes;
    int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    if (!x || !w || !y) return PT_ERR_NULL;
    IgemmArgs a{};
    a.A = x; a.B = w; a.D = y;
    a.M = d->N * d->P * d->Q; a.gH = d->P; a.gW = d->Q;
    a.srcH = d->H; a.srcW = d->W; a.apitch = d->x_cpitch;
    a.h_mul = d->stride_h; a.h_add = -d->pad_h; a.w_mul = d->stride_w; a.w_add = -d->pad_w;
    a.tr_step = 1; a.ts_step = 1; a.TR = d->R; a.TS = d->S;
    a.Cred = d->C; a.CredP = (int)round_up(d->C, 8);
    a.b_tap0 = 0; a.b_tr_stride = d->S; a.b_ts_stride = 1; a.b_taps = d->R * d->S;
    a.bpitch = d->w_cpitch; a.Nout = d->K;
    a.DH = d->P; a.DW = d->Q; a.d_hmul = 1; a.d_hadd = 0; a.d_wmul = 1; a.d_wadd = 0; a.dpitch = d->y_cpitch;
    a.a_vec = (d->x_cpitch % 8 == 0) && aligned16(x);
    a.b_vec = (d->w_cpitch % 8 == 0) && aligned16(w);
    a.d_vec = (d->y_cpitch % 4 == 0) && (((uintptr_t)y & 7) == 0);
    launch_igemm(a, (hipStream_t)stream);
    return launch_status();
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
    for (int ca = 0; ca < d->stride_h; ++ca) {
        for (int cb = 0; cb < d->stride_w; ++cb) {
            const int gH = ca < d->H ? (d->H - ca + d->stride_h - 1) / d->stride_h : 0;
            const int gW = cb < d->W ? (d->W - cb + d->stride_w - 1) / d->stride_w : 0;
            if (gH == 0 || gW == 0) continue;
            const int r0 = (ca + d->pad_h) % d->stride_h, s0 = (cb + d->pad_w) % d->stride_w;
            const int TR = r0 < d->R ? (d->R - r0 + d->stride_h - 1) / d->stride_h : 0;
            const int TS = s0 < d->S ? (d->S - s0 + d->stride_w - 1) / d->stride_w : 0;
            if (TR == 0 || TS == 0) {
                const int64_t pixels = (int64_t)d->N * gH * gW;
                const int64_t nblk = ceil_div(pixels * d->C, 256);
                if (nblk > 0x7fffffff) return PT_ERR_UNSUPPORTED;
                hipLaunchKernelGGL(k_zero_class, dim3((unsigned)nblk), dim3(256), 0, st, dx, pixels, gH, gW, d->H, d->W,
                                   d->stride_h, ca, d->stride_w, cb, d->x_cpitch, d->C);
            } else {
                IgemmArgs a{};
                a.A = dy; a.B = wt; a.D = dx;
                a.M = d->N * gH * gW; a.gH = gH; a.gW = gW;
                a.srcH = d->P; a.srcW = d->Q; a.apitch = d->y_cpitch;
                a.h_mul = 1; a.h_add = (ca + d->pad_h - r0) / d->stride_h;
                a.w_mul = 1; a.w_add = (cb + d->pad_w - s0) / d->stride_w;
                a.tr_step = -1; a.ts_step = -1; a.TR = TR; a.TS = TS;
                a.Cred = d->K; a.CredP = kpitch;
                a.b_tap0 = r0 * d->S + s0; a.b_tr_stride = d->stride_h * d->S; a.b_ts_stride = d->stride_w;
                a.b_taps = RS; a.bpitch = kpitch; a.Nout = d->C;
                a.DH = d->H; a.DW = d->W; a.d_hmul = d->stride_h; a.d_hadd = ca; a.d_wmul = d->stride_w; a.d_wadd = cb;
                a.dpitch = d->x_cpitch;
                a.a_vec = (d->y_cpitch % 8 == 0) && aligned16(dy);
                a.b_vec = 1;
                a.d_vec = (d->x_cpitch % 4 == 0) && (((uintptr_t)dx & 7) == 0);
                launch_igemm(a, st);
            }
            rc = launch_status();
            if (rc != PT_OK) return rc;
        }
    }
    return PT_OK;
}

extern "C" int32_t pt_conv_bwd_weight(const pt_conv_desc* d, const uint16_t* x, const uint16_t* dy, float* dw, void* ws,
                                      size_t ws_bytes, void* stream) {
    int32_t rc = check_desc(d);
    if (rc != PT_OK) return rc;
    if (!x || !dy || !dw) return PT_ERR_NULL;
    const WgradPlan p = plan_wgrad(d);
    if (p.ws_bytes > 0 && !ws) return PT_ERR_NULL;
    if (ws_bytes < p.ws_bytes) return PT_ERR_WORKSPACE;
    if (p.ws_bytes > 0 && !aligned16(ws)) return PT_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    WgradArgs a{};
    a.X = x; a.DY = dy;
    a.pixels = d->N * d->P * d->Q;
    a.P = d->P; a.Q = d->Q; a.H = d->H; a.W = d->W; a.xpitch = d->x_cpitch; a.ypitch = d->y_cpitch;
    a.magicQ = make_magic((uint32_t)d->Q); a.magicP = make_magic((uint32_t)d->P);
    a.stride_h = d->stride_h; a.stride_w = d->stride_w; a.pad_h = d->pad_h; a.pad_w = d->pad_w;
    a.S = d->S; a.RS = d->R * d->S; a.C = d->C; a.CP = p.CP; a.Mtot = p.Mtot; a.K = d->K;
    a.tiles_n = p.tiles_n;
    a.iters_total = p.iters_total; a.iters_per_split = p.iters_per_split; a.splits = p.splits;
    a.wpitch = d->w_cpitch;
    a.direct = p.splits == 1;
    a.OUT = a.direct ? dw : (float*)ws;
    a.out_row_pitch = p.Mtot;
    a.x_vec = (d->x_cpitch % 8 == 0) && aligned16(x);
    a.y_vec = (d->y_cpitch % 8 == 0) && aligned16(dy);
    a.o_vec = (d->w_cpitch % 4 == 0) && aligned16(dw);
    hipLaunchKernelGGL((k_wgrad<kWgBM, kWgBN, kWgBK, 2, 2>), dim3(p.tiles_m * p.tiles_n, p.splits), dim3(kConvThreads), 0,
                       st, a);
    rc = launch_status();
    if (rc != PT_OK) return rc;
    if (!a.direct) {
        const int64_t work = (int64_t)d->K * p.Mtot;
        const int64_t nblk = ceil_div(work, 256);
        if (nblk > 0x7fffffff) return PT_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(k_wgrad_reduce, dim3((unsigned)nblk), dim3(256), 0, st, (const float*)ws, p.splits, d->K, a.RS,
                           d->C, p.CP, d->w_cpitch, dw);
        rc = launch_status();
    }
    return rc;
}
