// Convolutions whose input has at most 4 channels (image stems, e.g. 7x7 stride 2 on RGB).
//
// With C = 3 an NHWC pixel is 6 bytes, so neither the 16-byte gathers of the general
// implicit-GEMM kernels nor their 64-deep contraction steps fit.  Here a workgroup copies the
// input patch under its 8x32 output tile into LDS once, padding every pixel to 4 halves
// (8 bytes).  One filter row then is a run of 8 padded pixels = 32 halves = two
// v_mfma_f32_32x32x16_f16 contraction steps, read straight from the patch:
//   forward : rows = filters (packed, zero-padded filter bank), columns = the 32 output
//             pixels of one tile row; a lane's operand is 2 adjacent padded pixels (16 bytes).
//   wgrad   : rows = filters (dy tile, transposing LDS read), columns = the 32 (s,c) slots of
//             one filter row (transposing LDS read of the patch: 4 consecutive output pixels
//             of one padded input pixel), contraction = output pixels along the tile row.
// Both are bound by the HBM traffic of the K-channel tensor (y or dy), so the y tile is
// written, and the dy tile read, as whole 128-byte lines.  A workgroup walks over several
// tiles and fetches the next tile's inputs into registers while it multiplies the current one.
#include "common.h"
#include "thin.h"

namespace sdconv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));

constexpr int kTH = 8, kTW = 32;        // output tile (rows x columns)
constexpr int kKT = 64;                 // filters per workgroup tile

__device__ __forceinline__ half4 lds_read_tr4(const unsigned char* p)
{
    typedef __attribute__((address_space(3))) short4v* lds_ptr;
    short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    return __builtin_bit_cast(half4, v);
}

// Packed filter bank for the forward pass:
//   Wp[kt][r][j][kk][e], kt = filter tile, j = 16-byte chunk 0..3 of the 32-half filter row,
//   kk = filter within the tile (64), e = half within the chunk; slot 8j+e = 4*s + c.
__global__ __launch_bounds__(256) void thin_pack_filter_kernel(const __half* __restrict__ w,
                                                              __half* __restrict__ wp, int K, int R, int S, int C,
                                                              long total)
{
    long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    int e = (int)(i & 7);
    long t = i >> 3;
    int kk = (int)(t % kKT); t /= kKT;
    int j = (int)(t & 3); t >>= 2;
    int r = (int)(t % R);
    int kt = (int)(t / R);
    int slot = 8 * j + e, s = slot >> 2, c = slot & 3, k = kt * kKT + kk;
    __half v = __half(0.f);
    if (k < K && s < S && c < C) v = w[(((long)k * R + r) * S + s) * C + c];
    wp[i] = v;
}

// The padded input patch of one output tile goes to LDS ([PH][PW] pixels of 8 bytes) in two
// halves: patch_fetch sends the loads of up to kPU pixels per thread, all of them in flight at
// once (unconditional loads from clamped addresses: a load under a branch would be waited for
// before the next one is sent), and patch_put writes them to LDS.  Between the two the caller
// multiplies the previous tile, so the latency of the loads is hidden.
constexpr int kPU = 6;                  // 256 threads x 6 pixels cover the 21 x 70 patch of a 7x7 stride-2 stem
typedef uint2v PatchRegs[kPU];      // (channels 0-1, channels 2-3) of the pixels a thread carries

__device__ __forceinline__ void patch_fetch(const ThinParams& P, int n, int ho0, int wo0, int tid, int first,
                                            PatchRegs& r)
{
    const unsigned short* X = reinterpret_cast<const unsigned short*>(P.X);
    const int h0 = ho0 * P.sh - P.ph, w0 = wo0 * P.sw - P.pw;
    const int total = P.PH * P.PW;
    const int c1 = P.C > 1 ? 1 : 0, c2 = P.C > 2 ? 2 : 0, c3 = P.C > 3 ? 3 : 0;
#pragma unroll
    for (int u = 0; u < kPU; ++u) {
        const int idx = first + tid + 256 * u;
        const int prow = idx / P.PW, pcol = idx - prow * P.PW;
        const int h = h0 + prow, w = w0 + pcol;
        const bool ok = idx < total && (unsigned)h < (unsigned)P.H && (unsigned)w < (unsigned)P.W;
        const unsigned short* px = X + (ok ? (((long)n * P.H + h) * P.W + w) * P.C : 0);
        const unsigned v0 = px[0], v1 = px[c1], v2 = px[c2], v3 = px[c3];
        unsigned lo = v0 | (c1 ? v1 << 16 : 0u);
        unsigned hi = (c2 ? v2 : 0u) | (c3 ? v3 << 16 : 0u);
        r[u].x = ok ? lo : 0u;
        r[u].y = ok ? hi : 0u;
    }
}

__device__ __forceinline__ void patch_put(const ThinParams& P, unsigned char* patch, int tid, int first,
                                          const PatchRegs& r)
{
    const int total = P.PH * P.PW;
#pragma unroll
    for (int u = 0; u < kPU; ++u) {
        const int idx = first + tid + 256 * u;
        if (idx < total) *reinterpret_cast<uint2v*>(patch + idx * 8) = r[u];
    }
}

// Pixels of the patch beyond the first 256 * kPU (filters or strides larger than a stem's).
__device__ __forceinline__ void patch_rest(const ThinParams& P, unsigned char* patch, int n, int ho0, int wo0, int tid)
{
    for (int first = 256 * kPU; first < P.PH * P.PW; first += 256 * kPU) {
        PatchRegs t;
        patch_fetch(P, n, ho0, wo0, tid, first, t);
        patch_put(P, patch, tid, first, t);
    }
}

__device__ __forceinline__ void tile_origin(const ThinParams& P, int tile, int& n, int& ho0, int& wo0)
{
    const int tw = tile % P.tiles_w;
    tile /= P.tiles_w;
    const int th = tile % P.tiles_h;
    n = tile / P.tiles_h;
    ho0 = th * kTH;
    wo0 = tw * kTW;
}

__global__ __launch_bounds__(256) void thin_fwd_kernel(ThinParams P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* ldsW = smem;                                   // [R][4][64] x 16 B
    unsigned char* patch = ldsW + P.R * 4 * kKT * 16;             // [PH][PW] x 8 B
    unsigned char* stage = patch + ((P.PH * P.PW * 8 + 15) & ~15);   // [256 pixels][128 B], chunk-swizzled

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;

    const int kt = blockIdx.y;
    {   // this filter tile's packed bank: R*4*64 chunks of 16 bytes, copied as is
        const uint4v* src = reinterpret_cast<const uint4v*>(P.Wp) + (long)kt * P.R * 4 * kKT;
        for (int i = tid; i < P.R * 4 * kKT; i += 256) reinterpret_cast<uint4v*>(ldsW)[i] = src[i];
    }

    PatchRegs pr;
    if ((int)blockIdx.x < P.ntiles) {
        int n, ho0, wo0;
        tile_origin(P, blockIdx.x, n, ho0, wo0);
        patch_fetch(P, n, ho0, wo0, tid, 0, pr);
    }
    for (int tile = blockIdx.x; tile < P.ntiles; tile += gridDim.x) {
        int n, ho0, wo0;
        tile_origin(P, tile, n, ho0, wo0);

        __syncthreads();                       // previous tile fully consumed
        patch_put(P, patch, tid, 0, pr);
        patch_rest(P, patch, n, ho0, wo0, tid);
        __syncthreads();
        if (tile + (int)gridDim.x < P.ntiles) {    // the next tile's patch travels while this one is multiplied
            int n2, ho2, wo2;
            tile_origin(P, tile + gridDim.x, n2, ho2, wo2);
            patch_fetch(P, n2, ho2, wo2, tid, 0, pr);
        }

        float16v acc[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

        for (int r = 0; r < P.R; ++r) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                half8 fa[2], fb[2];
#pragma unroll
                for (int row = 0; row < 2; ++row) {
                    int prow = (2 * wave + row) * P.sh + r;
                    int pcol = l32 * P.sw + 4 * q + 2 * lhi;
                    const unsigned char* src = patch + (prow * P.PW + pcol) * 8;
                    half4 p0 = *reinterpret_cast<const half4*>(src);
                    half4 p1 = *reinterpret_cast<const half4*>(src + 8);
                    fa[row] = __builtin_shufflevector(p0, p1, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
                    fb[kb] = *reinterpret_cast<const half8*>(ldsW + (((r * 4 + q * 2 + lhi) * kKT) + kb * 32 + l32) * 16);
#pragma unroll
                for (int row = 0; row < 2; ++row)
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
                        acc[row][kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[kb], fa[row], acc[row][kb], 0, 0, 0);
            }
        }

        // fp32 -> fp16 into the staging tile: pixel-major rows of 64 filters (128 bytes)
#pragma unroll
        for (int row = 0; row < 2; ++row) {
            int pix = (2 * wave + row) * kTW + l32;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    int k = kb * 32 + 8 * q + 4 * lhi;
                    float v[4] = {acc[row][kb][4 * q + 0], acc[row][kb][4 * q + 1], acc[row][kb][4 * q + 2],
                                  acc[row][kb][4 * q + 3]};
                    if (P.ep.any()) {
                        const int ho = ho0 + pix / kTW, wo = wo0 + pix % kTW;
                        if (ho < P.Ho && wo < P.Wo) {
                            const long o = (((long)n * P.Ho + ho) * P.Wo + wo) * P.K;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const int kk = kt * kKT + k + e;
                                if (kk < P.K) v[e] = epilogue_apply(P.ep, v[e], kk, o + kk);
                            }
                        }
                    }
                    half4 h;
                    h[0] = (_Float16)v[0];
                    h[1] = (_Float16)v[1];
                    h[2] = (_Float16)v[2];
                    h[3] = (_Float16)v[3];
                    int chunk = (k >> 3) ^ (pix & 7);
                    *reinterpret_cast<half4*>(stage + pix * 128 + chunk * 16 + (k & 7) * 2) = h;
                }
        }
        __syncthreads();
        // whole 128-byte lines out: 8 lanes per pixel
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int c = tid + 256 * i;
            int pix = c >> 3, part = c & 7;
            int ho = ho0 + pix / kTW, wo = wo0 + pix % kTW;
            int k = kt * kKT + part * 8;
            if (ho < P.Ho && wo < P.Wo && k < P.K) {
                uint4v v = *reinterpret_cast<const uint4v*>(stage + pix * 128 + ((part ^ (pix & 7)) << 4));
                __builtin_nontemporal_store(v, reinterpret_cast<uint4v*>(P.Y + ((((long)n * P.Ho + ho) * P.Wo + wo) * P.K + k)));
            }
        }
    }
}

// Weight gradient: every workgroup accumulates over the tiles it owns and writes one fp32
// partial [64 filters][R][32 slots] to the workspace; thin_wgrad_reduce_kernel adds them up.
__global__ __launch_bounds__(256) void thin_wgrad_kernel(ThinParams P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* gt = smem;                                   // dy tile [256 pixels][64 filters] halves
    unsigned char* patch = smem + kTH * kTW * kKT * 2;          // [PH][PW] x 8 B

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int grp = lane >> 4, gl = lane & 15;
    const int kt = blockIdx.y;

    // wave `wave` owns filter rows r = wave and wave + 4 (when they exist), both 32-filter blocks
    float16v acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

    // dy tile: 256 pixels x 128 bytes, 8 lanes per pixel; like the patch it is fetched into
    // registers one tile ahead and written to LDS when the previous tile has been multiplied
    auto dy_fetch = [&](int n, int ho0, int wo0, uint4v (&gv)[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = tid + 256 * i;
            const int pix = c >> 3, part = c & 7;
            const int ho = ho0 + pix / kTW, wo = wo0 + pix % kTW;
            const int k = kt * kKT + part * 8;
            const bool ok = ho < P.Ho && wo < P.Wo && k < P.K;
            const uint4v* src = reinterpret_cast<const uint4v*>(
                P.G + (ok ? (((long)n * P.Ho + ho) * P.Wo + wo) * P.K + k : 0));
            const uint4v v = *src;
            const uint4v z = {0u, 0u, 0u, 0u};
            gv[i] = ok ? v : z;
        }
    };
    PatchRegs pr;
    uint4v gv[8];
    if ((int)blockIdx.x < P.ntiles) {
        int n, ho0, wo0;
        tile_origin(P, blockIdx.x, n, ho0, wo0);
        patch_fetch(P, n, ho0, wo0, tid, 0, pr);
        dy_fetch(n, ho0, wo0, gv);
    }
    for (int tile = blockIdx.x; tile < P.ntiles; tile += gridDim.x) {
        int n, ho0, wo0;
        tile_origin(P, tile, n, ho0, wo0);

        __syncthreads();
        patch_put(P, patch, tid, 0, pr);
        patch_rest(P, patch, n, ho0, wo0, tid);
        // 64-byte granules of a dy row swizzled by pixel parity
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = tid + 256 * i;
            const int pix = c >> 3, part = c & 7;
            const int gran = (part >> 2) ^ (pix & 1);
            *reinterpret_cast<uint4v*>(gt + pix * 128 + gran * 64 + (part & 3) * 16) = gv[i];
        }
        __syncthreads();
        if (tile + (int)gridDim.x < P.ntiles) {
            int n2, ho2, wo2;
            tile_origin(P, tile + gridDim.x, n2, ho2, wo2);
            patch_fetch(P, n2, ho2, wo2, tid, 0, pr);
            dy_fetch(n2, ho2, wo2, gv);
        }

        for (int row = 0; row < kTH; ++row) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {                  // 16 output pixels per MFMA
                // filters x pixels operand from the dy tile
                half8 fa[2];
                const int pl = row * kTW + kk * 16 + 8 * (grp >> 1) + (gl >> 2);   // pixel of first read
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    int col = kb * 32 + 16 * (grp & 1) + 4 * (gl & 3);             // filter index
                    int byte = col * 2;
                    const unsigned char* a0 = gt + pl * 128 + (((byte >> 6) ^ (pl & 1)) << 6) + (byte & 63);
                    const unsigned char* a1 = gt + (pl + 4) * 128 + (((byte >> 6) ^ ((pl + 4) & 1)) << 6) + (byte & 63);
                    half4 lo = lds_read_tr4(a0), hi = lds_read_tr4(a1);
                    fa[kb] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int ri = 0; ri < 2; ++ri) {
                    int r = wave + 4 * ri;
                    if (r < P.R) {
                        // pixels x slots operand from the patch: slot 4s+c, lane 4i+j -> pixel i, s = 4*(grp&1)+j
                        int wo_l = kk * 16 + 8 * (grp >> 1) + (gl >> 2);
                        int s = 4 * (grp & 1) + (gl & 3);
                        const unsigned char* b0 = patch + ((row * P.sh + r) * P.PW + wo_l * P.sw + s) * 8;
                        half4 lo = lds_read_tr4(b0), hi = lds_read_tr4(b0 + 4 * P.sw * 8);
                        half8 fb = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                        for (int kb = 0; kb < 2; ++kb)
                            acc[ri][kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[kb], fb, acc[ri][kb], 0, 0, 0);
                    }
                }
            }
        }
    }

    // partial[wg][kt][k 0..63][r][slot 0..31]
    float* out = P.partial + ((long)blockIdx.x * gridDim.y + kt) * kKT * P.R * 32;
#pragma unroll
    for (int ri = 0; ri < 2; ++ri) {
        int r = wave + 4 * ri;
        if (r >= P.R) continue;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                int k = kb * 32 + 8 * (e >> 2) + 4 * lhi + (e & 3);
                out[(k * P.R + r) * 32 + l32] = acc[ri][kb][e];
            }
    }
}

// dw[k][r][s][c] = sum over workgroups of partial[wg][kt][kk][r][4s+c], fixed order.
// One block per (k, r): 32 slots x 8 partial-lanes.
__global__ __launch_bounds__(256) void thin_wgrad_reduce_kernel(const float* __restrict__ partial,
                                                               float* __restrict__ dw, int nwg, int ktiles,
                                                               int K, int R, int S, int C)
{
    __shared__ float red[8][32];
    const int k = blockIdx.x / R, r = blockIdx.x % R;
    const int kt = k / kKT, kk = k % kKT;
    const int slot = threadIdx.x & 31, part = threadIdx.x >> 5;
    // four independent chains so that four loads are in flight per thread; the order of the
    // additions depends on nwg only
    const long pitch = (long)ktiles * kKT * R * 32;
    const float* src = partial + (((long)kt * kKT + kk) * R + r) * 32 + slot;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int wg = part;
    for (; wg + 24 < nwg; wg += 32) {
        s0 += src[(long)wg * pitch];
        s1 += src[(long)(wg + 8) * pitch];
        s2 += src[(long)(wg + 16) * pitch];
        s3 += src[(long)(wg + 24) * pitch];
    }
    for (; wg < nwg; wg += 8) s0 += src[(long)wg * pitch];
    const float s = (s0 + s1) + (s2 + s3);
    red[part][slot] = s;
    __syncthreads();
    if (part == 0) {
        float tot = red[0][slot];
#pragma unroll
        for (int i = 1; i < 8; ++i) tot += red[i][slot];
        int sx = slot >> 2, c = slot & 3;
        if (sx < S && c < C) dw[(((long)k * R + r) * S + sx) * C + c] = tot;
    }
}

// Data gradient for C <= 4 on the vector ALU (v_dot2_f32_f16): the output has too few
// channels for a matrix tile.  One lane per dx pixel, lanes of a wave walk along w inside one
// stride-parity class, so the taps are wave-uniform and a wave reads 64 consecutive dy pixels
// (whole 128-byte lines) per tap.  The filter, re-laid-out as WT[C][R][S][K], sits in LDS and
// is read with uniform (broadcast) addresses.  KC = 16-byte chunks of K handled per inner step.
template <int KC>
__global__ __launch_bounds__(256) void thin_dgrad_kernel(ThinDgradParams P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int RS = P.R * P.S;
    {
        const uint4v* src = reinterpret_cast<const uint4v*>(P.WT);
        const int chunks = P.C * RS * P.K / 8;
        for (int i = threadIdx.x; i < chunks; i += 256) reinterpret_cast<uint4v*>(smem)[i] = src[i];
    }
    __syncthreads();
    const half8* wlds = reinterpret_cast<const half8*>(smem);

    int blk = blockIdx.x, cls = 0;
    while (cls + 1 < P.nclasses && blk >= P.class_block_start[cls + 1]) ++cls;
    blk -= P.class_block_start[cls];
    const int ca = cls / P.sw, cb = cls % P.sw;
    const int Hi = (P.H - ca + P.sh - 1) / P.sh, Wj = (P.W - cb + P.sw - 1) / P.sw;
    const int Mc = P.N * Hi * Wj;
    const int m = blk * 256 + threadIdx.x;
    const bool live = m < Mc;
    int n = 0, i = 0, j = 0;
    if (live) {
        n = m / (Hi * Wj);
        int rem = m - n * (Hi * Wj);
        i = rem / Wj;
        j = rem - i * Wj;
    }
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const int kchunks = P.K / 8;
    for (int r = 0; r < P.R; ++r) {
        const int th = ca + P.ph - r * P.dh;
        if (th % P.sh) continue;
        const int ho = i + th / P.sh;
        for (int s = 0; s < P.S; ++s) {
            const int tw = cb + P.pw - s * P.dw;
            if (tw % P.sw) continue;
            const int wo = j + tw / P.sw;
            const bool ok = live && (unsigned)ho < (unsigned)P.Ho && (unsigned)wo < (unsigned)P.Wo;
            const half8* gp = reinterpret_cast<const half8*>(P.G + (((long)n * P.Ho + ho) * P.Wo + wo) * P.K);
            const int tap = r * P.S + s;
            for (int kc0 = 0; kc0 < kchunks; kc0 += KC) {
                half8 g[KC];
#pragma unroll
                for (int u = 0; u < KC; ++u) {
                    half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
                    g[u] = z;
                    if (ok) g[u] = gp[kc0 + u];
                }
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (c < P.C) {
                        const half8* wp = wlds + ((c * RS + tap) * kchunks + kc0);
                        float a = acc[c];
#pragma unroll
                        for (int u = 0; u < KC; ++u) {
                            const half8 wv = wp[u];
                            a = __builtin_amdgcn_fdot2(g[u].s01, wv.s01, a, false);
                            a = __builtin_amdgcn_fdot2(g[u].s23, wv.s23, a, false);
                            a = __builtin_amdgcn_fdot2(g[u].s45, wv.s45, a, false);
                            a = __builtin_amdgcn_fdot2(g[u].s67, wv.s67, a, false);
                        }
                        acc[c] = a;
                    }
                }
            }
        }
    }
    if (live) {
        const long o = (((long)n * P.H + (ca + P.sh * i)) * P.W + (cb + P.sw * j)) * P.C;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (c < P.C) P.DX[o + c] = __float2half_rn(epilogue_apply(P.ep, acc[c], c, o + c));
    }
}

size_t thin_dgrad_lds_bytes(const Geom& g) { return (size_t)g.C * g.R * g.S * g.K * 2; }

hipError_t launch_thin_dgrad(const Geom& g, const __half* dy, const __half* wT, __half* dx, hipStream_t st,
                             const Epilogue& ep)
{
    ThinDgradParams P;
    P.ep = ep;
    P.G = dy; P.WT = wT; P.DX = dx;
    P.N = g.N; P.H = g.H; P.W = g.W; P.C = g.C; P.K = g.K; P.R = g.R; P.S = g.S;
    P.sh = g.sh; P.sw = g.sw; P.ph = g.ph; P.pw = g.pw; P.dh = g.dh; P.dw = g.dw; P.Ho = g.Ho; P.Wo = g.Wo;
    P.nclasses = g.sh * g.sw;
    int acc = 0;
    for (int q = 0; q < P.nclasses; ++q) {
        int a = q / g.sw, b = q % g.sw;
        long Hi = (g.H - a + g.sh - 1) / g.sh, Wj = (g.W - b + g.sw - 1) / g.sw;
        if (Hi < 0) Hi = 0;
        if (Wj < 0) Wj = 0;
        P.class_block_start[q] = acc;
        acc += (int)(((long)g.N * Hi * Wj + 255) / 256);
    }
    P.class_block_start[P.nclasses] = acc;
    size_t lds = thin_dgrad_lds_bytes(g);
    if (g.K % 64 == 0) hipLaunchKernelGGL(thin_dgrad_kernel<8>, dim3(acc), dim3(256), lds, st, P);
    else hipLaunchKernelGGL(thin_dgrad_kernel<1>, dim3(acc), dim3(256), lds, st, P);
    return hipGetLastError();
}

size_t thin_packed_filter_bytes(const Geom& g)
{
    int ktiles = (g.K + kKT - 1) / kKT;
    return (size_t)ktiles * g.R * 4 * kKT * 16;
}

// Workgroups walk over the tiles with a stride of the grid size: the grid is the smallest one
// that gives every workgroup the same number of tiles (2100 tiles on 512 resident workgroups:
// 420 workgroups of 5 tiles, not 512 of which a tenth take a fifth tile while the rest wait).
static int balanced_grid(int ntiles, int resident)
{
    const int per_wg = (ntiles + resident - 1) / resident;
    return (ntiles + per_wg - 1) / per_wg;
}

int thin_wgrad_workgroups(const Geom& g)
{
    int ntiles = g.N * ((g.Ho + kTH - 1) / kTH) * ((g.Wo + kTW - 1) / kTW);
    return balanced_grid(ntiles, 512);
}

size_t thin_wgrad_partial_bytes(const Geom& g)
{
    int ktiles = (g.K + kKT - 1) / kKT;
    return (size_t)thin_wgrad_workgroups(g) * ktiles * kKT * g.R * 32 * sizeof(float);
}

static ThinParams make_params(const Geom& g)
{
    ThinParams P;
    P.X = nullptr; P.Wp = nullptr; P.Y = nullptr; P.G = nullptr; P.partial = nullptr;
    P.N = g.N; P.H = g.H; P.W = g.W; P.C = g.C; P.K = g.K; P.R = g.R; P.S = g.S;
    P.sh = g.sh; P.sw = g.sw; P.ph = g.ph; P.pw = g.pw; P.Ho = g.Ho; P.Wo = g.Wo;
    P.tiles_h = (g.Ho + kTH - 1) / kTH;
    P.tiles_w = (g.Wo + kTW - 1) / kTW;
    P.ntiles = g.N * P.tiles_h * P.tiles_w;
    P.PH = (kTH - 1) * g.sh + g.R;
    P.PW = ((kTW - 1) * g.sw + 8 + 1) & ~1;
    return P;
}

bool thin_supported(const Geom& g)
{
    if (g.C > 4 || g.S > 8 || g.R > 8 || g.dh != 1 || g.dw != 1 || g.K % 8) return false;
    ThinParams P = make_params(g);
    size_t fwd_lds = (size_t)g.R * 4 * kKT * 16 + (((size_t)P.PH * P.PW * 8 + 15) & ~(size_t)15) + 256 * 128;
    return fwd_lds <= 150 * 1024;
}

hipError_t launch_thin_fwd(const Geom& g, const __half* x, const __half* w, __half* y, void* ws, hipStream_t st,
                           const Epilogue& ep)
{
    ThinParams P = make_params(g);
    int ktiles = (g.K + kKT - 1) / kKT;
    __half* wp = static_cast<__half*>(ws);
    long total = (long)ktiles * g.R * 4 * kKT * 8;
    hipLaunchKernelGGL(thin_pack_filter_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       w, wp, g.K, g.R, g.S, g.C, total);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    P.X = x; P.Wp = wp; P.Y = y;
    P.ep = ep;
    size_t lds = (size_t)g.R * 4 * kKT * 16 + (((size_t)P.PH * P.PW * 8 + 15) & ~(size_t)15) + 256 * 128;
    static std::atomic<bool> configured{false};   // set once the attribute call has succeeded; a second thread may repeat it, harmlessly
    if (!configured.load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&thin_fwd_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    const int grid = balanced_grid(P.ntiles, 512);     // two workgroups per compute unit fit in LDS
    hipLaunchKernelGGL(thin_fwd_kernel, dim3(grid, ktiles), dim3(256), lds, st, P);
    return hipGetLastError();
}

hipError_t launch_thin_wgrad(const Geom& g, const __half* x, const __half* dy, float* dw, void* ws, hipStream_t st)
{
    ThinParams P = make_params(g);
    int ktiles = (g.K + kKT - 1) / kKT;
    int nwg = thin_wgrad_workgroups(g);
    P.X = x; P.G = dy; P.partial = static_cast<float*>(ws);
    size_t lds = (size_t)kTH * kTW * kKT * 2 + (size_t)P.PH * P.PW * 8;
    hipError_t e;
    static std::atomic<bool> configured{false};   // set once the attribute call has succeeded; a second thread may repeat it, harmlessly
    if (!configured.load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&thin_wgrad_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(thin_wgrad_kernel, dim3(nwg, ktiles), dim3(256), lds, st, P);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(thin_wgrad_reduce_kernel, dim3(g.K * g.R), dim3(256), 0, st,
                       static_cast<const float*>(ws), dw, nwg, ktiles, g.K, g.R, g.S, g.C);
    return hipGetLastError();
}

}  // namespace sdconv
