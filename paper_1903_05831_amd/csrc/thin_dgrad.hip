// Data gradient of a strided convolution with at most 4 input channels (image stems) on MFMA.
//
// The stride-parity classes of dx are merged into one stride-1 problem over "macro pixels":
// macro pixel (i,j) holds the sh*sw dx pixels (i*sh+a, j*sw+b), i.e. sh*sw*4 output slots
// (a,b,c) <= 16.  Class (a,b) sees filter tap r only if a + pad - r*dil is a multiple of the
// stride, and then reads dy row i + oh with oh = (a + pad - r*dil)/stride; over all classes oh
// spans a small window [ohmin, ohmin+RP), likewise ow.  A merged filter
//     Wm[(r',s')][k][slot]  (zero where a class has no tap at that displacement)
// turns the whole data gradient into a dense RP x SP stride-1 convolution from K channels to 16
// slots:  rows = slots (A operand, held in registers for the whole workgroup), columns = 16
// consecutive macro pixels (B operand, read from a dy patch in LDS), v_mfma_f32_16x16x32_f16.
// Each lane ends up with the <= 4 channels of one dx pixel.  The kernel is bound by reading dy
// (whole 128-byte lines via LDS-DMA, zeros outside the image from the range check).
#include "common.h"
#include "thin.h"
#include "dma.h"

namespace sdconv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kDI = 8, kDJ = 32;      // macro-pixel tile (rows x columns)
constexpr int kMaxMergedTaps = 16;

__global__ __launch_bounds__(256) void thin_dgrad_merge_filter_kernel(
    const __half* __restrict__ w, __half* __restrict__ wm, ThinDgradMfmaParams P, int total)
{
    int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int e = idx & 7, t0 = idx >> 3;
    int slot = t0 & 15; t0 >>= 4;
    int kchunks = P.K / 8;
    int kc = t0 % kchunks, t = t0 / kchunks;
    int k = kc * 8 + e;
    int cls = slot >> 2, c = slot & 3;
    int a = cls / P.sw, b = cls % P.sw;
    int oh = t / P.SP + P.ohmin, ow = t % P.SP + P.owmin;
    __half v = __half(0.f);
    if (cls < P.sh * P.sw && c < P.C) {
        int nr = a + P.ph - P.sh * oh, ns = b + P.pw - P.sw * ow;
        if (nr >= 0 && ns >= 0 && nr % P.dh == 0 && ns % P.dw == 0) {
            int r = nr / P.dh, s = ns / P.dw;
            if (r < P.R && s < P.S) v = w[(((long)k * P.R + r) * P.S + s) * P.C + c];
        }
    }
    wm[idx] = v;
}

template <int KQ>   // K / 32
__global__ __launch_bounds__(256) void thin_dgrad_mfma_kernel(ThinDgradMfmaParams P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    int t = blockIdx.x;
    const int tj = t % P.tiles_j; t /= P.tiles_j;
    const int ti = t % P.tiles_i;
    const int n = t / P.tiles_i;
    const int i0 = ti * kDI, j0 = tj * kDJ;
    const int PH = kDI + P.RP - 1, PW = kDJ + P.SP - 1;
    const int npix = PH * PW;

    // ---- dy patch -> LDS: 8 pixels (128 bytes each) per wave instruction, chunk-swizzled ----
    const int4v rsrcG = make_rsrc(P.G, (unsigned)(P.N * P.Ho * P.Wo * P.K) * 2u);
    for (int base = wave * 8; base < npix; base += 32) {
        int p = base + (lane >> 3);
        unsigned voff = kOutOfRange;
        if (p < npix) {
            int prow = p / PW, pcol = p - prow * PW;
            int ho = i0 + P.ohmin + prow, wo = j0 + P.owmin + pcol;
            int lc = (lane & 7) ^ ((p >> 1) & 7);
            if ((unsigned)ho < (unsigned)P.Ho && (unsigned)wo < (unsigned)P.Wo && lc * 8 < P.K)
                voff = (unsigned)(((((n * P.Ho + ho) * P.Wo + wo) * P.K) + lc * 8) * 2);
        }
        dma16(voff, rsrcG, 0, lds0 + base * 128);
    }

    // ---- merged filter -> registers (A operand: row = slot, 8 consecutive k per lane) --------
    const int ntm = P.RP * P.SP;
    const int kchunks = P.K / 8;
    half8 fw[kMaxMergedTaps][KQ];
    const half8* wm = reinterpret_cast<const half8*>(P.Wm);
#pragma unroll
    for (int tt = 0; tt < kMaxMergedTaps; ++tt)
#pragma unroll
        for (int q = 0; q < KQ; ++q) {
            half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
            fw[tt][q] = z;
            if (tt < ntm) fw[tt][q] = wm[(tt * kchunks + 4 * q + (lane >> 4)) * 16 + (lane & 15)];
        }

    wait_vmcnt<0>();
    __syncthreads();

    const int ncol = lane & 15, kq = lane >> 4;
    const int cls = kq, ca = cls / P.sw, cb = cls % P.sw;
#pragma unroll 1
    for (int gi = 0; gi < 4; ++gi) {
        const int g = wave * 4 + gi;
        const int ii = g >> 1, jseg = (g & 1) * 16;
        float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int tt = 0; tt < kMaxMergedTaps; ++tt) {
            if (tt < ntm) {
                const int rp = tt / P.SP, sp = tt - rp * P.SP;
                const int p = (ii + rp) * PW + jseg + ncol + sp;
#pragma unroll
                for (int q = 0; q < KQ; ++q) {
                    const int chunk = (4 * q + kq) ^ ((p >> 1) & 7);
                    half8 fb = *reinterpret_cast<const half8*>(smem + p * 128 + (chunk << 4));
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw[tt][q], fb, acc, 0, 0, 0);
                }
            }
        }
        const int h = (i0 + ii) * P.sh + ca, w = (j0 + jseg + ncol) * P.sw + cb;
        if (cls < P.sh * P.sw && h < P.H && w < P.W) {
            const long o = (((long)n * P.H + h) * P.W + w) * P.C;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (c < P.C) P.DX[o + c] = __float2half_rn(epilogue_apply(P.ep, acc[c], c, o + c));
        }
    }
}

static bool merged_window(int stride, int pad, int dil, int R, int* omin, int* ext)
{
    int lo = 1 << 30, hi = -(1 << 30);
    for (int a = 0; a < stride; ++a)
        for (int r = 0; r < R; ++r) {
            int th = a + pad - r * dil;
            if (th % stride) continue;
            int o = th / stride;
            if (o < lo) lo = o;
            if (o > hi) hi = o;
        }
    if (lo > hi) return false;
    *omin = lo;
    *ext = hi - lo + 1;
    return true;
}

static bool make_mfma_params(const Geom& g, ThinDgradMfmaParams* P)
{
    if (g.C > 4 || g.sh * g.sw > 4 || (g.K != 32 && g.K != 64)) return false;
    if (!merged_window(g.sh, g.ph, g.dh, g.R, &P->ohmin, &P->RP)) return false;
    if (!merged_window(g.sw, g.pw, g.dw, g.S, &P->owmin, &P->SP)) return false;
    if (P->RP * P->SP > kMaxMergedTaps) return false;
    P->N = g.N; P->H = g.H; P->W = g.W; P->C = g.C; P->K = g.K; P->R = g.R; P->S = g.S;
    P->sh = g.sh; P->sw = g.sw; P->ph = g.ph; P->pw = g.pw; P->dh = g.dh; P->dw = g.dw;
    P->Ho = g.Ho; P->Wo = g.Wo;
    P->tiles_i = ((g.H + g.sh - 1) / g.sh + kDI - 1) / kDI;
    P->tiles_j = ((g.W + g.sw - 1) / g.sw + kDJ - 1) / kDJ;
    return true;
}

static size_t mfma_lds_bytes(const ThinDgradMfmaParams& P)
{
    int npix = (kDI + P.RP - 1) * (kDJ + P.SP - 1);
    return (size_t)((npix + 31) / 32 * 32) * 128;
}

bool thin_dgrad_mfma_supported(const Geom& g)
{
    ThinDgradMfmaParams P;
    return make_mfma_params(g, &P) && mfma_lds_bytes(P) <= 64 * 1024;
}

size_t thin_dgrad_mfma_workspace_bytes(const Geom& g)
{
    ThinDgradMfmaParams P;
    if (!make_mfma_params(g, &P)) return 0;
    return (size_t)P.RP * P.SP * g.K * 16 * sizeof(__half);
}

hipError_t launch_thin_dgrad_mfma(const Geom& g, const __half* dy, const __half* w, __half* dx, void* ws,
                                  hipStream_t st, const Epilogue& ep)
{
    ThinDgradMfmaParams P;
    if (!make_mfma_params(g, &P)) return hipErrorInvalidValue;
    P.ep = ep;
    __half* wm = static_cast<__half*>(ws);
    P.G = dy; P.Wm = wm; P.DX = dx;
    int total = P.RP * P.SP * g.K * 16;
    hipLaunchKernelGGL(thin_dgrad_merge_filter_kernel, dim3((total + 255) / 256), dim3(256), 0, st, w, wm, P, total);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    size_t lds = mfma_lds_bytes(P);
    int grid = g.N * P.tiles_i * P.tiles_j;
    if (g.K == 64) hipLaunchKernelGGL(thin_dgrad_mfma_kernel<2>, dim3(grid), dim3(256), lds, st, P);
    else hipLaunchKernelGGL(thin_dgrad_mfma_kernel<1>, dim3(grid), dim3(256), lds, st, P);
    return hipGetLastError();
}

}  // namespace sdconv
