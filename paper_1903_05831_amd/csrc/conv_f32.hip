// Single-precision companion of the convolution path: the same three passes on binary32
// tensors with v_mfma_f32_32x32x2_f32 (binary32 products, binary32 accumulation).  It exists so
// that the FP32 -> FP16 speedup of section 2.2 / Figure 1(b) of the paper can be measured on this
// hardware with both sides on the matrix cores.
//
// The fp32 matrix rate is 1/16 of the fp16 one (157.3 against 2516.6 TFLOP/s), so these
// kernels are bound by the matrix pipe with a wide margin: a 128x128 tile needs 16 KB of
// operands per 2048 cycles of MFMA.  They therefore keep the plain structure of igemm.hip /
// wgrad.hip (global -> registers -> LDS double buffer, one barrier per step) and spend no
// effort on the memory side.
//
// Forward / data gradient: implicit GEMM, rows = pixels, 32 floats of contraction per step (a
// 128-byte row, 16-byte chunks XOR-swizzled with the row number).  An MFMA takes one float per
// lane and operand: lane l supplies row l%32 at contraction slot l/32.  A lane reads the 16-byte
// chunk 2j + l/32 of its row and uses its four floats in four consecutive MFMAs; the filter
// operand does the same, so both sides agree on which contraction index sits in which slot.
// The data gradient contracts over a transposed copy wT[c][r][s][k] of the filter (workspace).
//
// Weight gradient: rows = filters, columns = channels of one tap, contraction = pixels, 32 per
// step, tiles kept [pixel][channel] as they sit in memory: lane l reads channel l%32 of pixel
// 2t + l/32 with a 4-byte LDS read (odd pixel rows are stored with their columns XOR 32, which
// puts the two pixel rows of one read on different banks).  Split along the pixels, partial
// sums added in a fixed order by the reduction kernel of wgrad.hip.
#include "common.h"
#include "igemm.h"
#include "wgrad.h"

namespace sdconv {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct F32Params {
    const float* A;
    const float* B;
    float* D;
    int NB, Hs, Ws, Cs, Hd, Wd, Cd, R, S;
    int sh, sw, ph, pw, dh, dw;
    int nclasses, sw_cls, tiles_n, total_tiles, b_row_pitch;
    int class_tile_start[kMaxClasses + 1];
};

constexpr int kF32BK = 32;              // contraction floats per step
constexpr int kF32RowBytes = kF32BK * 4;

template <int MODE, int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void igemm_f32_kernel(F32Params P)
{
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int PA = BM / 32, PB = BN / 32;       // staging passes (32 rows per pass)
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is a multiple of the MFMA block");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* ldsA = smem;                                 // [2][BM rows][128 B]
    unsigned char* ldsB = smem + 2 * BM * kF32RowBytes;         // [2][BN rows][128 B]
    int* tap_oh = reinterpret_cast<int*>(smem + 2 * (BM + BN) * kF32RowBytes);
    int* tap_ow = tap_oh + kMaxTaps;
    int* tap_bo = tap_ow + kMaxTaps;
    int* tap_cnt = tap_bo + kMaxTaps;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    const int tile = blockIdx.x;
    const int tn = tile % P.tiles_n;
    int tm = tile / P.tiles_n;
    int cls = 0;
    while (cls + 1 < P.nclasses && tm >= P.class_tile_start[cls + 1]) ++cls;
    tm -= P.class_tile_start[cls];
    const int ca = cls / P.sw_cls, cb = cls % P.sw_cls;   // stride parity class (data gradient) or (0,0)

    int Hi, Wj, mh, mw, eh, ew;
    if (MODE == 0) { Hi = P.Hd; Wj = P.Wd; mh = P.sh; mw = P.sw; eh = 1; ew = 1; }
    else {
        Hi = (P.Hd - ca + P.sh - 1) / P.sh; Wj = (P.Wd - cb + P.sw - 1) / P.sw;
        mh = 1; mw = 1; eh = P.sh; ew = P.sw;
    }
    const int Mcls = P.NB * Hi * Wj;
    const int m0 = tm * BM, n0 = tn * BN;

    if (wave == 0) {
        const int ntap_all = P.R * P.S;
        bool ok = false;
        int oh = 0, ow = 0;
        const int r = lane / P.S, s = lane % P.S;
        if (lane < ntap_all) {
            if (MODE == 0) { ok = true; oh = r * P.dh - P.ph; ow = s * P.dw - P.pw; }
            else {
                int th = ca + P.ph - r * P.dh, tw = cb + P.pw - s * P.dw;
                ok = (th % P.sh == 0) && (tw % P.sw == 0);
                oh = th / P.sh; ow = tw / P.sw;
            }
        }
        unsigned long long mask = __ballot(ok);
        int pos = __popcll(mask & ((1ull << lane) - 1ull));
        if (ok) { tap_oh[pos] = oh; tap_ow[pos] = ow; tap_bo[pos] = (r * P.S + s) * P.Cs; }
        if (lane == 0) tap_cnt[0] = __popcll(mask);
    }
    __syncthreads();
    const int ntaps = __builtin_amdgcn_readfirstlane(tap_cnt[0]);
    const int kchunks = (P.Cs + kF32BK - 1) / kF32BK;
    const int nk = ntaps * kchunks;

    const int lrow = tid >> 3;        // 0..31
    const int kc = tid & 7;           // 16-byte chunk (4 floats) within the 128-byte row
    int a_base[PA], a_ih[PA], a_jw[PA];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        int m = m0 + lrow + 32 * p;
        if (m < Mcls) {
            int n = m / (Hi * Wj);
            int rem = m - n * (Hi * Wj);
            int i = rem / Wj, j = rem - i * Wj;
            a_base[p] = n * P.Hs * P.Ws * P.Cs;
            a_ih[p] = i * mh;
            a_jw[p] = j * mw;
        } else {
            a_base[p] = 0; a_ih[p] = -(1 << 28); a_jw[p] = -(1 << 28);
        }
    }
    int b_base[PB];
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        int n = n0 + lrow + 32 * p;
        b_base[p] = (n < P.Cd) ? n * P.b_row_pitch : -1;
    }

    f32x4 ra[PA], rb[PB];
    auto prefetch = [&](int it) {
        const int t = it / kchunks;
        const int c = (it - t * kchunks) * kF32BK + kc * 4;
        const int oh = tap_oh[t], ow = tap_ow[t], bo = tap_bo[t];
        const bool cok = c < P.Cs;                 // Cs is a multiple of 4: all four floats or none
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            int hs = a_ih[p] + oh, ws = a_jw[p] + ow;
            bool ok = cok && (unsigned)hs < (unsigned)P.Hs && (unsigned)ws < (unsigned)P.Ws;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (ok) v = *reinterpret_cast<const f32x4*>(P.A + (a_base[p] + (hs * P.Ws + ws) * P.Cs + c));
            ra[p] = v;
        }
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            bool ok = cok && b_base[p] >= 0;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (ok) v = *reinterpret_cast<const f32x4*>(P.B + (b_base[p] + bo + c));
            rb[p] = v;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            int row = lrow + 32 * p;
            *reinterpret_cast<f32x4*>(ldsA + buf * BM * kF32RowBytes + row * kF32RowBytes + ((kc ^ (row & 7)) << 4)) = ra[p];
        }
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            int row = lrow + 32 * p;
            *reinterpret_cast<f32x4*>(ldsB + buf * BN * kF32RowBytes + row * kF32RowBytes + ((kc ^ (row & 7)) << 4)) = rb[p];
        }
    };

    f32x16 acc[FN][FM];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

    const int l32 = lane & 31, lhi = lane >> 5;
    auto compute = [&](int buf) {
        const unsigned char* sa = ldsA + buf * BM * kF32RowBytes;
        const unsigned char* sb = ldsB + buf * BN * kF32RowBytes;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int chunk = 2 * j + lhi;          // contraction floats 4*chunk .. 4*chunk+3 of the step
            f32x4 fa[FM], fb[FN];
#pragma unroll
            for (int b = 0; b < FM; ++b) {
                int row = wm * WM + b * 32 + l32;
                fa[b] = *reinterpret_cast<const f32x4*>(sa + row * kF32RowBytes + ((chunk ^ (row & 7)) << 4));
            }
#pragma unroll
            for (int a = 0; a < FN; ++a) {
                int row = wn * WN + a * 32 + l32;
                fb[a] = *reinterpret_cast<const f32x4*>(sb + row * kF32RowBytes + ((chunk ^ (row & 7)) << 4));
            }
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int a = 0; a < FN; ++a)
#pragma unroll
                    for (int b = 0; b < FM; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fb[a][t], fa[b][t], acc[a][b], 0, 0, 0);
        }
    };

    if (nk > 0) {
        prefetch(0);
        stage(0);
        __syncthreads();
        for (int it = 0; it < nk; ++it) {
            const bool more = it + 1 < nk;
            if (more) prefetch(it + 1);
            compute(it & 1);
            if (more) stage((it + 1) & 1);
            __syncthreads();
        }
    }

    // ---- epilogue: a lane holds 4 consecutive destination channels of one pixel per group ----
#pragma unroll
    for (int b = 0; b < FM; ++b) {
        int m = m0 + wm * WM + b * 32 + l32;
        if (m >= Mcls) continue;
        int n = m / (Hi * Wj);
        int rem = m - n * (Hi * Wj);
        int i = rem / Wj, j = rem - i * Wj;
        int hd = i * eh + ca, wd = j * ew + cb;
        float* drow = P.D + ((long)(n * P.Hd + hd) * P.Wd + wd) * P.Cd;
#pragma unroll
        for (int a = 0; a < FN; ++a) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int col = n0 + wn * WN + a * 32 + 8 * q + 4 * lhi;
                if (col < P.Cd) {                   // Cd is a multiple of 4
                    f32x4 v = {acc[a][b][4 * q + 0], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]};
                    *reinterpret_cast<f32x4*>(drow + col) = v;
                }
            }
        }
    }
}

// wT[c][r][s][k] = w[k][r][s][c]
__global__ __launch_bounds__(256) void filter_transpose_f32_kernel(const float* __restrict__ w, float* __restrict__ wT,
                                                                   int K, int RS, int C)
{
    __shared__ float tile[32][33];
    const int tap = blockIdx.z;
    const int k0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int i = ty; i < 32; i += 8) {
        int k = k0 + i, c = c0 + tx;
        tile[i][tx] = (k < K && c < C) ? w[((long)k * RS + tap) * C + c] : 0.f;
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        int c = c0 + i, k = k0 + tx;
        if (c < C && k < K) wT[((long)c * RS + tap) * K + k] = tile[tx][i];
    }
}

// ---- weight gradient ---------------------------------------------------------------------------
struct F32WgradParams {
    const float* X;
    const float* G;
    float* out;             // dw when splits == 1, else [splits][K][R][S][C]
    int N, H, W, C, K, R, S;
    int sh, sw, ph, pw, dh, dw;
    int Ho, Wo, P;
    int splits, steps_per_split;    // pixel ranges, 32-pixel steps each covers
    int tiles_k, tiles_c;
};

constexpr int kF32BP = 32;          // pixels per contraction step

template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void wgrad_f32_kernel(F32WgradParams P)
{
    static_assert(WGM * WGN == 4, "four waves");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int TA = BM / 4, TB = BN / 4;                 // threads per tile row (16 B each)
    constexpr int PA = kF32BP * TA / 256, PB = kF32BP * TB / 256;
    constexpr int RA = 256 / TA, RB = 256 / TB;             // rows per pass
    static_assert(PA >= 1 && PB >= 1 && WM % 32 == 0 && WN % 32 == 0, "tile shape");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* ldsG = reinterpret_cast<float*>(smem);                            // [2][32][BM]
    float* ldsX = reinterpret_cast<float*>(smem) + 2 * kF32BP * BM;          // [2][32][BN]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    int b = blockIdx.x;
    const int tc = b % P.tiles_c; b /= P.tiles_c;
    const int tk = b % P.tiles_k; b /= P.tiles_k;
    const int tap = b % (P.R * P.S);
    const int split = b / (P.R * P.S);
    const int r = tap / P.S, s = tap % P.S;
    const int k0 = tk * BM, c0 = tc * BN;
    const int oh = r * P.dh - P.ph, ow = s * P.dw - P.pw;

    const int step0 = split * P.steps_per_split;
    int nsteps = (P.P + kF32BP - 1) / kF32BP - step0;
    if (nsteps > P.steps_per_split) nsteps = P.steps_per_split;

    const int ga_row = tid / TA, ga_col = (tid % TA) * 4;
    const int xb_row = tid / TB, xb_col = (tid % TB) * 4;
    const bool ga_ok = k0 + ga_col < P.K;                   // K and C are multiples of 4
    const bool xb_ok = c0 + xb_col < P.C;

    f32x4 rg[PA], rx[PB];
    auto prefetch = [&](int step) {
        const int p0 = (step0 + step) * kF32BP;
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            int p = p0 + ga_row + i * RA;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (ga_ok && p < P.P) v = *reinterpret_cast<const f32x4*>(P.G + ((long)p * P.K + k0 + ga_col));
            rg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            int p = p0 + xb_row + i * RB;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (xb_ok && p < P.P) {
                int n = p / (P.Ho * P.Wo);
                int rem = p - n * (P.Ho * P.Wo);
                int ho = rem / P.Wo, wo = rem - ho * P.Wo;
                int h = ho * P.sh + oh, w = wo * P.sw + ow;
                if ((unsigned)h < (unsigned)P.H && (unsigned)w < (unsigned)P.W)
                    v = *reinterpret_cast<const f32x4*>(P.X + ((((long)n * P.H + h) * P.W + w) * P.C + c0 + xb_col));
            }
            rx[i] = v;
        }
    };
    // odd pixel rows keep their columns XOR 32: the two rows one fragment read touches then lie
    // on different banks
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            int row = ga_row + i * RA;
            *reinterpret_cast<f32x4*>(ldsG + (buf * kF32BP + row) * BM + (ga_col ^ ((row & 1) << 5))) = rg[i];
        }
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            int row = xb_row + i * RB;
            *reinterpret_cast<f32x4*>(ldsX + (buf * kF32BP + row) * BN + (xb_col ^ ((row & 1) << 5))) = rx[i];
        }
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][c][e] = 0.f;

    const int l32 = lane & 31, lhi = lane >> 5;
    auto compute = [&](int buf) {
#pragma unroll
        for (int t = 0; t < kF32BP / 2; ++t) {
            const int row = 2 * t + lhi;            // pixel of the step: parity == lhi
            const float* sg = ldsG + (buf * kF32BP + row) * BM;
            const float* sx = ldsX + (buf * kF32BP + row) * BN;
            float fa[FM], fb[FN];
#pragma unroll
            for (int a = 0; a < FM; ++a) fa[a] = sg[(wm * WM + a * 32 + l32) ^ (lhi << 5)];
#pragma unroll
            for (int c = 0; c < FN; ++c) fb[c] = sx[(wn * WN + c * 32 + l32) ^ (lhi << 5)];
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int c = 0; c < FN; ++c)
                    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a], fb[c], acc[a][c], 0, 0, 0);
        }
    };

    if (nsteps > 0) {
        prefetch(0);
        stage(0);
        __syncthreads();
        for (int it = 0; it < nsteps; ++it) {
            const bool more = it + 1 < nsteps;
            if (more) prefetch(it + 1);
            compute(it & 1);
            if (more) stage((it + 1) & 1);
            __syncthreads();
        }
    }

    const long numel = (long)P.K * P.R * P.S * P.C;
    float* out = P.out + (long)split * numel;
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c) {
            int col = c0 + wn * WN + c * 32 + l32;
            if (col >= P.C) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                int k = k0 + wm * WM + a * 32 + 8 * (e >> 2) + 4 * lhi + (e & 3);
                if (k < P.K) out[((long)k * P.R * P.S + tap) * P.C + col] = acc[a][c][e];
            }
        }
}

// ---- host side -----------------------------------------------------------------------------------
static size_t f32_align256(size_t b) { return (b + 255) & ~(size_t)255; }

bool f32_supported(const Geom& g)
{
    return g.C % 4 == 0 && g.K % 4 == 0 && g.R * g.S <= kMaxTaps && g.sh * g.sw <= kMaxClasses;
}

static void f32_wgrad_shape(const Geom& g, int* bm, int* bn, int* splits, int* sps)
{
    *bm = g.K <= 64 ? 64 : 128;
    *bn = g.C <= 64 ? 64 : 128;
    const long tiles = (long)((g.K + *bm - 1) / *bm) * ((g.C + *bn - 1) / *bn) * g.R * g.S;
    const long total_steps = ((long)g.N * g.Ho * g.Wo + kF32BP - 1) / kF32BP;
    // enough pixel ranges for two workgroups per compute unit, in whole multiples of the unit count
    long cap = total_steps / 8;
    if (cap < 1) cap = 1;
    long want = 1;
    double best = -1.0;
    for (long sp = 1; sp <= cap && sp * tiles <= 2048; ++sp) {
        const long wgs = sp * tiles;
        const double fill = (double)wgs / (double)(((wgs + 255) / 256) * 256);
        const double enough = wgs >= 512 ? 1.0 : (double)wgs / 512.0;
        const double score = fill * enough - 1e-5 * sp;         // ties: fewer partial sums
        if (score > best) { best = score; want = sp; }
    }
    const long per = (total_steps + want - 1) / want;
    *sps = (int)per;
    *splits = (int)((total_steps + per - 1) / per);
}

size_t f32_workspace_bytes(const Geom& g, int pass)
{
    if (!f32_supported(g)) return 0;
    if (pass == SDCONV_DGRAD) return f32_align256((size_t)g.K * g.R * g.S * g.C * sizeof(float));
    if (pass == SDCONV_WGRAD) {
        int bm, bn, splits, sps;
        f32_wgrad_shape(g, &bm, &bn, &splits, &sps);
        return splits > 1 ? f32_align256((size_t)splits * g.K * g.R * g.S * g.C * sizeof(float)) : 0;
    }
    return 0;
}

template <int MODE, int BM, int BN, int WGM, int WGN>
static hipError_t launch_f32_variant(const F32Params& P, hipStream_t st)
{
    constexpr size_t lds = 2 * (BM + BN) * kF32RowBytes + (3 * kMaxTaps + 4) * sizeof(int);
    static std::atomic<bool> configured{false};   // set once the attribute call has succeeded; a second thread may repeat it, harmlessly
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_f32_kernel<MODE, BM, BN, WGM, WGN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((igemm_f32_kernel<MODE, BM, BN, WGM, WGN>), dim3(P.total_tiles), dim3(256), lds, st, P);
    return hipGetLastError();
}

static hipError_t run_f32_igemm(const Geom& g, bool dgrad, const float* A, const float* B, float* D, hipStream_t st)
{
    F32Params P;
    P.A = A; P.B = B; P.D = D;
    P.NB = g.N;
    if (!dgrad) { P.Hs = g.H; P.Ws = g.W; P.Cs = g.C; P.Hd = g.Ho; P.Wd = g.Wo; P.Cd = g.K; }
    else        { P.Hs = g.Ho; P.Ws = g.Wo; P.Cs = g.K; P.Hd = g.H; P.Wd = g.W; P.Cd = g.C; }
    P.R = g.R; P.S = g.S;
    P.sh = g.sh; P.sw = g.sw; P.ph = g.ph; P.pw = g.pw; P.dh = g.dh; P.dw = g.dw;
    P.sw_cls = dgrad ? g.sw : 1;
    P.b_row_pitch = g.R * g.S * P.Cs;
    // Tile: 128x128, 128x64 or 64x64, chosen below (these kernels are matrix-bound, so an idle or
    // overloaded compute unit costs its full share).
    auto count_tiles = [&](int bm, int bn, bool fill) {
        int acc = 0;
        if (!dgrad) {
            if (fill) { P.nclasses = 1; P.class_tile_start[0] = 0; }
            acc = (int)(((long)g.N * g.Ho * g.Wo + bm - 1) / bm);
            if (fill) P.class_tile_start[1] = acc;
        } else {
            const int nc = g.sh * g.sw;
            if (fill) P.nclasses = nc;
            for (int q = 0; q < nc; ++q) {
                int a = q / g.sw, b = q % g.sw;
                long Hi = (g.H - a + g.sh - 1) / g.sh, Wj = (g.W - b + g.sw - 1) / g.sw;
                if (Hi < 0) Hi = 0;
                if (Wj < 0) Wj = 0;
                if (fill) P.class_tile_start[q] = acc;
                acc += (int)((g.N * Hi * Wj + bm - 1) / bm);
            }
            if (fill) P.class_tile_start[nc] = acc;
        }
        return (long)acc * ((P.Cd + bn - 1) / bn);
    };
    // score = how evenly the tiles spread over the compute units (they are all resident at once and
    // share the matrix pipes: the fullest unit sets the time) x a small preference for the larger tile
    const int cus = 256;
    const int cand[3][2] = {{128, 128}, {128, 64}, {64, 64}};
    const double pref[3] = {1.0, 0.96, 0.90};
    int bm = 64, bn = 64;
    double best = -1.0;
    for (int i = 0; i < 3; ++i) {
        if (cand[i][1] == 128 && P.Cd <= 64) continue;
        const long t = count_tiles(cand[i][0], cand[i][1], false);
        const double fill = (double)t / (double)(((t + cus - 1) / cus) * cus);
        if (fill * pref[i] > best) { best = fill * pref[i]; bm = cand[i][0]; bn = cand[i][1]; }
    }
    P.tiles_n = (P.Cd + bn - 1) / bn;
    P.total_tiles = (int)count_tiles(bm, bn, true);
    if (P.total_tiles <= 0) return hipErrorInvalidValue;
    if (bm == 64) return dgrad ? launch_f32_variant<1, 64, 64, 2, 2>(P, st) : launch_f32_variant<0, 64, 64, 2, 2>(P, st);
    if (bn == 64) return dgrad ? launch_f32_variant<1, 128, 64, 2, 2>(P, st) : launch_f32_variant<0, 128, 64, 2, 2>(P, st);
    return dgrad ? launch_f32_variant<1, 128, 128, 2, 2>(P, st) : launch_f32_variant<0, 128, 128, 2, 2>(P, st);
}

hipError_t run_fwd_f32(const Geom& g, const float* x, const float* w, float* y, hipStream_t st)
{
    if (!f32_supported(g)) return launch_direct_fwd_f32(g, x, w, y, st);
    return run_f32_igemm(g, false, x, w, y, st);
}

hipError_t run_dgrad_f32(const Geom& g, const float* dy, const float* w, float* dx, void* ws, hipStream_t st)
{
    if (!f32_supported(g)) return launch_direct_dgrad_f32(g, dy, w, dx, st);
    float* wT = static_cast<float*>(ws);
    dim3 grid((g.C + 31) / 32, (g.K + 31) / 32, g.R * g.S);
    hipLaunchKernelGGL(filter_transpose_f32_kernel, grid, dim3(256), 0, st, w, wT, g.K, g.R * g.S, g.C);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return run_f32_igemm(g, true, dy, wT, dx, st);
}

template <int BM, int BN>
static hipError_t launch_f32_wgrad(const F32WgradParams& P, hipStream_t st)
{
    constexpr size_t lds = 2 * kF32BP * (BM + BN) * sizeof(float);
    static std::atomic<bool> configured{false};   // set once the attribute call has succeeded; a second thread may repeat it, harmlessly
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_f32_kernel<BM, BN, 2, 2>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    long blocks = (long)P.tiles_c * P.tiles_k * P.R * P.S * P.splits;
    hipLaunchKernelGGL((wgrad_f32_kernel<BM, BN, 2, 2>), dim3((unsigned)blocks), dim3(256), lds, st, P);
    return hipGetLastError();
}

hipError_t run_wgrad_f32(const Geom& g, const float* x, const float* dy, float* dw, void* ws, hipStream_t st)
{
    if (!f32_supported(g)) return launch_direct_wgrad_f32(g, x, dy, dw, st);
    F32WgradParams P;
    int bm, bn;
    f32_wgrad_shape(g, &bm, &bn, &P.splits, &P.steps_per_split);
    P.X = x; P.G = dy;
    P.N = g.N; P.H = g.H; P.W = g.W; P.C = g.C; P.K = g.K; P.R = g.R; P.S = g.S;
    P.sh = g.sh; P.sw = g.sw; P.ph = g.ph; P.pw = g.pw; P.dh = g.dh; P.dw = g.dw;
    P.Ho = g.Ho; P.Wo = g.Wo;
    P.P = g.N * g.Ho * g.Wo;
    P.tiles_k = (g.K + bm - 1) / bm;
    P.tiles_c = (g.C + bn - 1) / bn;
    P.out = P.splits > 1 ? static_cast<float*>(ws) : dw;
    hipError_t e;
    if (bm == 128 && bn == 128) e = launch_f32_wgrad<128, 128>(P, st);
    else if (bm == 128) e = launch_f32_wgrad<128, 64>(P, st);
    else if (bn == 128) e = launch_f32_wgrad<64, 128>(P, st);
    else e = launch_f32_wgrad<64, 64>(P, st);
    if (e != hipSuccess || P.splits == 1) return e;
    return launch_splitk_reduce(static_cast<const float*>(ws), dw, P.splits, (long)g.K * g.R * g.S * g.C, st);
}

}  // namespace sdconv
