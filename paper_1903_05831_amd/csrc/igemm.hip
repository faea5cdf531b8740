// Implicit-GEMM convolution on fp16 MFMA for gfx950: forward and data gradient.
//
// Both passes are "gather rows of an activation tensor, multiply by a filter matrix whose
// rows are contiguous along the contraction":
//   forward : D = y,  A = x,  B = w  [K][R][S][C]        (contraction runs over r,s,c)
//   dgrad   : D = dx, A = dy, B = wT [C][R][S][K]        (contraction runs over r,s,k)
// The im2col matrix is never formed: each thread keeps, for the tile rows it loads, the
// decoded pixel coordinates and tests every filter tap against the image border when it
// issues the 16-byte NHWC load (zero-fill outside).
//
// Strided dgrad is split by output parity: pixels with (h mod stride_h, w mod stride_w) =
// (a,b) form one class, and a class only sees the taps whose offset has that parity, so no
// multiply is spent on structural zeros.  A class without taps writes zeros.
//
// Tiling: 256 threads = 4 waves per workgroup; a BM(pixels) x BN(filters) tile, contraction
// step 64 halves (one 128-byte line per pixel); global -> VGPR -> LDS double buffer with one
// barrier per step; LDS rows are 128 bytes with their 16-byte chunks XOR-swizzled by the row
// number so that both the staging writes and the MFMA fragment reads are conflict-free;
// v_mfma_f32_32x32x16_f16 with the filter fragment as the row operand, which leaves every
// lane with 4 consecutive output channels of one pixel (an 8-byte NHWC store).
#include "common.h"
#include "igemm.h"

namespace sdconv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;            // contraction halves per step
constexpr int kRowBytes = kBK * 2; // 128
constexpr int kThreads = 256;

// MODE 0: forward (rows are output pixels, source = x).  MODE 1: data gradient (rows are
// input pixels of one parity class, source = dy).
template <int MODE, int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(kThreads) void igemm_kernel(IgemmParams P)
{
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;       // 32x32 MFMA blocks per wave
    constexpr int PA = BM / 32, PB = BN / 32;       // staging passes (32 rows per pass)
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is a multiple of the MFMA block");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // [2][BM rows][128 B] then [2][BN rows][128 B], then the tap table
    unsigned char* ldsA = smem;
    unsigned char* ldsB = smem + 2 * BM * kRowBytes;
    int* tap_oh = reinterpret_cast<int*>(smem + 2 * (BM + BN) * kRowBytes);
    int* tap_ow = tap_oh + kMaxTaps;
    int* tap_bo = tap_ow + kMaxTaps;
    int* tap_cnt = tap_bo + kMaxTaps;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    // ---- which tile -------------------------------------------------------------
    const int tile = blockIdx.x;
    const int tn = tile % P.tiles_n;
    int tm = tile / P.tiles_n;
    int cls = 0;
    while (cls + 1 < P.nclasses && tm >= P.class_tile_start[cls + 1]) ++cls;
    tm -= P.class_tile_start[cls];
    const int ca = cls / P.sw_cls, cb = cls % P.sw_cls;   // parity class (dgrad) or (0,0)

    int Hi, Wj, mh, mw, eh, ew;
    if (MODE == 0) { Hi = P.Hd; Wj = P.Wd; mh = P.sh; mw = P.sw; eh = 1; ew = 1; }
    else {
        Hi = (P.Hd - ca + P.sh - 1) / P.sh; Wj = (P.Wd - cb + P.sw - 1) / P.sw;
        mh = 1; mw = 1; eh = P.sh; ew = P.sw;
    }
    const int Mcls = P.NB * Hi * Wj;
    const int m0 = tm * BM, n0 = tn * BN;

    // ---- tap table (one wave builds it) --------------------------------------------
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
    const int kchunks = (P.Cs + kBK - 1) / kBK;
    const int nk = ntaps * kchunks;

    // ---- per-thread staging rows -----------------------------------------------------
    const int lrow = tid >> 3;        // 0..31
    const int kc = tid & 7;           // 16-byte chunk within the 128-byte row
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

    uint4v ra[PA], rb[PB];
    auto prefetch = [&](int it) {
        const int t = it / kchunks;
        const int c = (it - t * kchunks) * kBK + kc * 8;
        const int oh = tap_oh[t], ow = tap_ow[t], bo = tap_bo[t];
        const bool cok = c < P.Cs;
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            int hs = a_ih[p] + oh, ws = a_jw[p] + ow;
            bool ok = cok && (unsigned)hs < (unsigned)P.Hs && (unsigned)ws < (unsigned)P.Ws;
            uint4v v = {0u, 0u, 0u, 0u};
            if (ok) v = *reinterpret_cast<const uint4v*>(P.A + (a_base[p] + (hs * P.Ws + ws) * P.Cs + c));
            ra[p] = v;
        }
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            bool ok = cok && b_base[p] >= 0;
            uint4v v = {0u, 0u, 0u, 0u};
            if (ok) v = *reinterpret_cast<const uint4v*>(P.B + (b_base[p] + bo + c));
            rb[p] = v;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            int row = lrow + 32 * p;
            *reinterpret_cast<uint4v*>(ldsA + buf * BM * kRowBytes + row * kRowBytes + ((kc ^ (row & 7)) << 4)) = ra[p];
        }
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            int row = lrow + 32 * p;
            *reinterpret_cast<uint4v*>(ldsB + buf * BN * kRowBytes + row * kRowBytes + ((kc ^ (row & 7)) << 4)) = rb[p];
        }
    };

    float16v acc[FN][FM];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

    const int l32 = lane & 31, lhi = lane >> 5;
    auto compute = [&](int buf) {
        const unsigned char* sa = ldsA + buf * BM * kRowBytes;
        const unsigned char* sb = ldsB + buf * BN * kRowBytes;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int chunk = kk * 2 + lhi;
            half8 fa[FM], fb[FN];
#pragma unroll
            for (int b = 0; b < FM; ++b) {
                int row = wm * WM + b * 32 + l32;
                fa[b] = *reinterpret_cast<const half8*>(sa + row * kRowBytes + ((chunk ^ (row & 7)) << 4));
            }
#pragma unroll
            for (int a = 0; a < FN; ++a) {
                int row = wn * WN + a * 32 + l32;
                fb[a] = *reinterpret_cast<const half8*>(sb + row * kRowBytes + ((chunk ^ (row & 7)) << 4));
            }
#pragma unroll
            for (int a = 0; a < FN; ++a)
#pragma unroll
                for (int b = 0; b < FM; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[a], fa[b], acc[a][b], 0, 0, 0);
        }
    };

    // ---- main loop ---------------------------------------------------------------------
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

    // ---- epilogue: fp32 -> fp16 (nearest even), 8-byte NHWC stores ----------------------------
#pragma unroll
    for (int b = 0; b < FM; ++b) {
        int m = m0 + wm * WM + b * 32 + l32;
        if (m >= Mcls) continue;
        int n = m / (Hi * Wj);
        int rem = m - n * (Hi * Wj);
        int i = rem / Wj, j = rem - i * Wj;
        int hd = i * eh + ca, wd = j * ew + cb;
        __half* drow = P.D + ((n * P.Hd + hd) * P.Wd + wd) * P.Cd;
#pragma unroll
        for (int a = 0; a < FN; ++a) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int col = n0 + wn * WN + a * 32 + 8 * q + 4 * lhi;
                if (col < P.Cd) {
                    half4 h;
                    const long o = (drow - P.D) + col;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        h[e] = (_Float16)epilogue_apply(P.ep, acc[a][b][4 * q + e], col + e, o + e);
                    *reinterpret_cast<half4*>(drow + col) = h;
                }
            }
        }
    }
}

// wT[c][r][s][k] = w[k][r][s][c]: the filter matrix of the data gradient, contraction-major.
__global__ __launch_bounds__(256) void filter_transpose_kernel(const __half* __restrict__ w,
                                                               __half* __restrict__ wT, int K, int RS, int C)
{
    __shared__ __half tile[32][33];
    const int tap = blockIdx.z;
    const int k0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int i = ty; i < 32; i += 8) {
        int k = k0 + i, c = c0 + tx;
        tile[i][tx] = (k < K && c < C) ? w[((long)k * RS + tap) * C + c] : __half(0.f);
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        int c = c0 + i, k = k0 + tx;
        if (c < C && k < K) wT[((long)c * RS + tap) * K + k] = tile[tx][i];
    }
}

template <int MODE, int BM, int BN, int WGM, int WGN>
static hipError_t launch_variant(const IgemmParams& P, int total_tiles, hipStream_t st)
{
    constexpr size_t lds = 2 * (BM + BN) * kRowBytes + (3 * kMaxTaps + 4) * sizeof(int);
    static std::atomic<bool> configured{false};   // set once the attribute call has succeeded; a second thread may repeat it, harmlessly
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_kernel<MODE, BM, BN, WGM, WGN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((igemm_kernel<MODE, BM, BN, WGM, WGN>), dim3(total_tiles), dim3(kThreads), lds, st, P);
    return hipGetLastError();
}

const IgemmVariant kIgemmVariants[kNumIgemmVariants] = {
    {128, 128, "igemm_fwd_128x128", "igemm_dgrad_128x128"},
    {256, 128, "igemm_fwd_256x128", "igemm_dgrad_256x128"},
    {256, 64, "igemm_fwd_256x64", "igemm_dgrad_256x64"},
    {128, 64, "igemm_fwd_128x64", "igemm_dgrad_128x64"},
};

hipError_t launch_igemm(int variant, const IgemmParams& P, int total_tiles, hipStream_t st)
{
    const int key = variant * 2 + (P.mode ? 1 : 0);
    switch (key) {
        case 0: return launch_variant<0, 128, 128, 2, 2>(P, total_tiles, st);
        case 1: return launch_variant<1, 128, 128, 2, 2>(P, total_tiles, st);
        case 2: return launch_variant<0, 256, 128, 2, 2>(P, total_tiles, st);
        case 3: return launch_variant<1, 256, 128, 2, 2>(P, total_tiles, st);
        case 4: return launch_variant<0, 256, 64, 4, 1>(P, total_tiles, st);
        case 5: return launch_variant<1, 256, 64, 4, 1>(P, total_tiles, st);
        case 6: return launch_variant<0, 128, 64, 2, 2>(P, total_tiles, st);
        case 7: return launch_variant<1, 128, 64, 2, 2>(P, total_tiles, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_filter_transpose(const __half* w, __half* wT, int K, int RS, int C, hipStream_t st)
{
    dim3 grid((C + 31) / 32, (K + 31) / 32, RS);
    hipLaunchKernelGGL(filter_transpose_kernel, grid, dim3(256), 0, st, w, wT, K, RS, C);
    return hipGetLastError();
}

}  // namespace sdconv
