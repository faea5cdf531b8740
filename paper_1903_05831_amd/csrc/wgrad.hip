// Weight gradient on fp16 MFMA for gfx950, split along the pixel (contraction) axis.
//
//   dw[k][r][s][c] = sum_p dy[p][k] * x[src(p; r,s)][c],   p = (n,ho,wo)
//
// GEMM view: rows = filters k (from dy), columns = channels c of one tap, contraction =
// output pixels.  Neither operand is contiguous along the contraction (NHWC keeps channels
// innermost), so tiles are staged in LDS exactly as they sit in memory -- [pixel][channel] --
// and the MFMA fragments are fetched with the transposing LDS read ds_read_b64_tr_b16, which
// hands each lane four consecutive pixels of one channel.
//
// One workgroup owns a (filter tile, channel tile, tap, pixel range) and walks its pixel
// range in steps of 64.  With more than one pixel range the fp32 tile goes to a workspace
// slice and a second kernel adds the slices in a fixed order (bit-reproducible).
#include "common.h"
#include "wgrad.h"

namespace sdconv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

constexpr int kBP = 64;   // pixels per contraction step
constexpr int kWThreads = 256;

// Four consecutive contraction rows of one column, for 16 lanes at a time.
__device__ __forceinline__ half4 lds_read_tr(const unsigned char* p)
{
    typedef __attribute__((address_space(3))) short4v* lds_ptr;
    short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    return __builtin_bit_cast(half4, v);
}

// Byte offset of (row, col half-index) in a [kBP][BW halves] tile whose 64-byte granules are
// XOR-swizzled with the row number inside each 256-byte group.
template <int BW>
__device__ __forceinline__ int tile_off(int row, int col)
{
    constexpr int pitch = BW * 2;
    int byte = col * 2;
    int gran = byte >> 6;
    constexpr int gmask = (pitch >= 256) ? 3 : (pitch / 64 - 1);
    gran ^= (row & gmask);
    return row * pitch + (gran << 6) + (byte & 63);
}

template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(kWThreads) void wgrad_kernel(WgradParams P)
{
    static_assert(WGM * WGN == 4, "four waves");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int TA = BM / 8, TB = BN / 8;               // threads per tile row (16 B each)
    constexpr int PA = kBP * TA / kWThreads, PB = kBP * TB / kWThreads;   // staging passes
    constexpr int RA = kWThreads / TA, RB = kWThreads / TB;               // rows per pass
    static_assert(PA >= 1 && PB >= 1, "tile too narrow for 256 threads");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* ldsG = smem;                               // [2][kBP][BM] halves
    unsigned char* ldsX = smem + 2 * kBP * BM * 2;            // [2][kBP][BN] halves

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
    int nsteps = (P.P + kBP - 1) / kBP - step0;
    if (nsteps > P.steps_per_split) nsteps = P.steps_per_split;

    // staging coordinates
    const int ga_row = tid / TA, ga_col = (tid % TA) * 8;     // dy tile
    const int xb_row = tid / TB, xb_col = (tid % TB) * 8;     // x tile
    const bool ga_ok = k0 + ga_col < P.K;
    const bool xb_ok = c0 + xb_col < P.C;

    uint4v rg[PA], rx[PB];
    auto prefetch = [&](int step) {
        const int p0 = (step0 + step) * kBP;
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            int p = p0 + ga_row + i * RA;
            uint4v v = {0u, 0u, 0u, 0u};
            if (ga_ok && p < P.P) v = *reinterpret_cast<const uint4v*>(P.G + ((long)p * P.K + k0 + ga_col));
            rg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            int p = p0 + xb_row + i * RB;
            uint4v v = {0u, 0u, 0u, 0u};
            if (xb_ok && p < P.P) {
                int n = p / (P.Ho * P.Wo);
                int rem = p - n * (P.Ho * P.Wo);
                int ho = rem / P.Wo, wo = rem - ho * P.Wo;
                int h = ho * P.sh + oh, w = wo * P.sw + ow;
                if ((unsigned)h < (unsigned)P.H && (unsigned)w < (unsigned)P.W)
                    v = *reinterpret_cast<const uint4v*>(P.X + ((((long)n * P.H + h) * P.W + w) * P.C + c0 + xb_col));
            }
            rx[i] = v;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PA; ++i)
            *reinterpret_cast<uint4v*>(ldsG + buf * kBP * BM * 2 + tile_off<BM>(ga_row + i * RA, ga_col)) = rg[i];
#pragma unroll
        for (int i = 0; i < PB; ++i)
            *reinterpret_cast<uint4v*>(ldsX + buf * kBP * BN * 2 + tile_off<BN>(xb_row + i * RB, xb_col)) = rx[i];
    };

    float16v acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][c][e] = 0.f;

    // Fragment addressing: 16-lane group g = lane/16 serves columns 16*(g&1).. of a 32-wide
    // block and contraction rows 8*(g>>1)..+8; inside the group lane 4i+j points at row i,
    // columns 4j..4j+3; two reads (rows +0..3 and +4..7) fill the 8-deep operand.
    const int grp = lane >> 4, gl = lane & 15;
    const int frag_row = 8 * (grp >> 1) + (gl >> 2);
    const int frag_col = 16 * (grp & 1) + 4 * (gl & 3);

    auto compute = [&](int buf) {
        const unsigned char* sg = ldsG + buf * kBP * BM * 2;
        const unsigned char* sx = ldsX + buf * kBP * BN * 2;
#pragma unroll
        for (int kk = 0; kk < kBP / 16; ++kk) {
            half8 fa[FM], fb[FN];
            const int row = kk * 16 + frag_row;
#pragma unroll
            for (int a = 0; a < FM; ++a) {
                int col = wm * WM + a * 32 + frag_col;
                half4 lo = lds_read_tr(sg + tile_off<BM>(row, col));
                half4 hi = lds_read_tr(sg + tile_off<BM>(row + 4, col));
                fa[a] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int c = 0; c < FN; ++c) {
                int col = wn * WN + c * 32 + frag_col;
                half4 lo = lds_read_tr(sx + tile_off<BN>(row, col));
                half4 hi = lds_read_tr(sx + tile_off<BN>(row + 4, col));
                fb[c] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int c = 0; c < FN; ++c)
                    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[a], fb[c], acc[a][c], 0, 0, 0);
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

    // ---- store the fp32 tile: lanes 0..31 hold consecutive channels of one filter row ------
    const long numel = (long)P.K * P.R * P.S * P.C;
    float* out = P.out + (long)split * numel;
    const int l32 = lane & 31, lhi = lane >> 5;
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

// dw[e] = sum over the splits of partial[k][e], in a fixed order: G groups of threads take the
// splits k = g, g+G, g+2G, ... of an element each (in that order), then group 0 adds the G
// group sums in group order.  G > 1 keeps small gradients with many splits from running on a
// handful of threads with a long serial chain of loads each; any G gives run-to-run identical
// results for a given (numel, splits), since G is a function of those two only.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial,
                                                            float* __restrict__ dw, int splits, long numel4, int G)
{
    __shared__ float4v sh[256];
    const int epb = 256 / G;                        // elements (of 4 floats) per block
    const int e = threadIdx.x % epb, g = threadIdx.x / epb;
    const long i = (long)blockIdx.x * epb + e;
    const float4v* p = reinterpret_cast<const float4v*>(partial);
    float4v s = {0.f, 0.f, 0.f, 0.f};
    if (i < numel4) {
        for (int k = g; k < splits; k += G) {
            float4v v = p[(long)k * numel4 + i];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
    }
    if (G > 1) {
        sh[threadIdx.x] = s;
        __syncthreads();
        if (g == 0) {
            for (int gg = 1; gg < G; ++gg) {
                float4v v = sh[gg * epb + e];
                s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
            }
        }
    }
    if (g == 0 && i < numel4) reinterpret_cast<float4v*>(dw)[i] = s;
}

template <int BM, int BN, int WGM, int WGN>
static hipError_t launch_wvariant(const WgradParams& P, hipStream_t st)
{
    constexpr size_t lds = 2 * kBP * (BM + BN) * 2;
    static std::atomic<bool> configured{false};   // set once the attribute call has succeeded; a second thread may repeat it, harmlessly
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_kernel<BM, BN, WGM, WGN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    long blocks = (long)P.tiles_c * P.tiles_k * P.R * P.S * P.splits;
    hipLaunchKernelGGL((wgrad_kernel<BM, BN, WGM, WGN>), dim3((unsigned)blocks), dim3(kWThreads), lds, st, P);
    return hipGetLastError();
}

const WgradVariant kWgradVariants[kNumWgradVariants] = {
    {128, 128, "wgrad_128x128"},
    {64, 128, "wgrad_64x128"},
};

hipError_t launch_wgrad(int variant, const WgradParams& P, hipStream_t st)
{
    switch (variant) {
        case 0: return launch_wvariant<128, 128, 2, 2>(P, st);
        case 1: return launch_wvariant<64, 128, 1, 4>(P, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_splitk_reduce(const float* partial, float* dw, int splits, long numel, hipStream_t st)
{
    long n4 = numel / 4;   // numel is a multiple of 64 on this route (C and K multiples of 8)
    int G = 1;
    while (G < 16 && G * 2 <= splits && n4 * G < 65536) G *= 2;
    const int epb = 256 / G;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n4 + epb - 1) / epb)), dim3(256), 0, st,
                       partial, dw, splits, n4, G);
    return hipGetLastError();
}

}  // namespace sdconv
