// Weight gradient with an asynchronous global->LDS pipeline (see wgrad.hip for the maths).
//
//   dw[k][r][s][c] = sum_p dy[p][k] * x[src(p; r,s)][c],   p = (n,ho,wo)
//
// One workgroup owns a (filter tile, channel tile, tap, pixel range).  Per contraction step
// it needs BP pixels of dy (rows of BM filters) and the BP matching pixels of x (rows of BN
// channels); both tiles go to LDS as they sit in memory, [pixel][channel], with
// buffer_load_dwordx4 ... lds into a ring of S stages, and the MFMA fragments come from the
// transposing LDS read (four consecutive pixels of one channel per lane).
//
// Addressing: dy rows are consecutive pixels, so a lane's offset is fixed and the buffer
// descriptor's base moves by BP rows per step; its shrinking size makes the hardware range
// check zero the rows past the last pixel.  x rows are gathered: BP lanes decode one pixel
// each per step into an LDS table of byte offsets (out-of-image -> out of range -> zeros), one
// step ahead of the loads that use it; with a 1x1 stride-1 unpadded filter x is addressed like
// dy and the table is skipped (LINEAR).
//
// 64-byte granules of a tile row are XOR-swizzled with the row number (applied on the global
// side by choosing which chunk a lane fetches) so the transposing reads are conflict-free.
#include <type_traits>
#include "common.h"
#include "wgrad.h"
#include "dma.h"

#include "lds_tr.h"

namespace sdconv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4w __attribute__((ext_vector_type(4)));

// HF: only the upper half of the waves sends the loads (and then multiplies like the others).
// With two waves per SIMD the lower wave keeps the matrix pipe busy while its partner is stalled
// in the burst of LDS-DMA instructions, instead of both stalling at once (see igemm_ws.hip).
// MF: 32 = v_mfma_f32_32x32x16_f16 blocks, 16 = v_mfma_f32_16x16x32_f16 blocks (measured faster
// on the large tiles).
template <int BM, int BN, int WGM, int WGN, int S, int BP, bool LINEAR, bool HF, int MF = 32>
__global__ __launch_bounds__(64 * WGM * WGN) void wgrad_dma_kernel(WgradParams P)
{
    constexpr int NW = WGM * WGN;
    constexpr int NWF = HF ? NW / 2 : NW, NT = 64 * NWF;    // fetching waves / threads
    constexpr int FW0 = NW - NWF;                           // first fetching wave
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / MF, FN = WN / MF;
    constexpr int ACCN = MF == 32 ? 16 : 4, KSTEP = MF == 32 ? 16 : 32;
    constexpr int CRG = BM / 8, CRX = BN / 8;           // 16-byte chunks per tile row
    constexpr int RPG = NT / CRG, RPX = NT / CRX;       // rows one pass of all threads covers
    constexpr int PG = BP / RPG, PX = BP / RPX;         // DMA loads per thread and stage
    constexpr int GBYTES = BP * BM * 2, XBYTES = BP * BN * 2, STAGE = GBYTES + XBYTES;
    constexpr int INFLIGHT = (S - 2) * (PG + PX);
    static_assert((MF == 32 || MF == 16) && WM % MF == 0 && WN % MF == 0 && BP % KSTEP == 0, "wave tile");
    static_assert(PG >= 1 && PX >= 1 && BP % RPG == 0 && BP % RPX == 0 && RPG % 4 == 0 && RPX % 4 == 0, "staging");
    static_assert(S >= 2 && INFLIGHT < 64 && BP % 16 == 0 && BP <= 64 * NW, "pipeline");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
    unsigned* xtab = reinterpret_cast<unsigned*>(smem + S * STAGE);     // [S][BP] byte offsets of x pixels

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const bool fetcher = wave >= FW0;
    const int ft = tid - FW0 * 64, fw = wave - FW0;         // index among the fetching threads / waves

    // Which tile: the tiles of one pixel range (all filter tiles, channel tiles and taps of a
    // split) read the same dy and x rows, and each XCD has an L2 of its own, so runs of 8
    // consecutive tiles go to one XCD (workgroup b runs on XCD b % 8) instead of being dealt round
    // over all eight, which made every XCD fetch every operand row again.
    constexpr int kRun = 8;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    int b = ((slot / kRun) * 8 + xcd) * kRun + (slot % kRun);
    if (b >= P.total_blocks) return;
    const int tc = b % P.tiles_c; b /= P.tiles_c;
    const int tk = b % P.tiles_k; b /= P.tiles_k;
    const int tap = b % (P.R * P.S);
    const int split = b / (P.R * P.S);
    const int r = tap / P.S, s = tap % P.S;
    const int k0 = tk * BM, c0 = tc * BN;
    const int oh = r * P.dh - P.ph, ow = s * P.dw - P.pw;

    const int bp_per_64 = 64 / BP;                           // steps_per_split counts 64-pixel units
    const int step0 = split * P.steps_per_split * bp_per_64;
    const int total_steps = (P.P + BP - 1) / BP;
    int nsteps = total_steps - step0;
    if (nsteps > P.steps_per_split * bp_per_64) nsteps = P.steps_per_split * bp_per_64;
    if (nsteps < 0) nsteps = 0;

    // ---- fixed per-thread parts of the offsets ----------------------------------------------
    unsigned g_off[PG], x_add[PX];
    int x_row[PX];
#pragma unroll
    for (int i = 0; i < PG; ++i) {
        int row = i * RPG + ft / CRG, pc = ft % CRG;
        int lc = swizzled_chunk<BM>(row, pc);
        int k = k0 + lc * 8;
        g_off[i] = (k < P.K) ? (unsigned)((row * P.K + k) * 2) : kOutOfRange;
    }
#pragma unroll
    for (int i = 0; i < PX; ++i) {
        int row = i * RPX + ft / CRX, pc = ft % CRX;
        int lc = swizzled_chunk<BN>(row, pc);
        int c = c0 + lc * 8;
        x_row[i] = row;
        if (LINEAR) x_add[i] = (c < P.C) ? (unsigned)((row * P.C + c) * 2) : kOutOfRange;
        else x_add[i] = (c < P.C) ? (unsigned)(c * 2) : kOutOfRange;
    }
    const int4v rsrcX = make_rsrc(P.X, (unsigned)(P.N * P.H * P.W * P.C) * 2u);

    // x offset table of one step: lane t < BP holds pixel p0 + t.  The steps come in order, so
    // the lane keeps its pixel's (image, row, column) and moves it on by BP pixels per step with
    // two carries instead of dividing again (the divisions cost 5 % of a 3x3 layer's kernel).
    int tb_p = 0, tb_n = 0, tb_ho = 0, tb_wo = 0;
    const int hw = P.Ho * P.Wo;
    const int adv_n = BP / hw, adv_ho = (BP % hw) / P.Wo, adv_wo = (BP % hw) % P.Wo;
    if (!LINEAR && tid < BP) {
        tb_p = step0 * BP + tid;
        tb_n = tb_p / hw;
        const int rem = tb_p - tb_n * hw;
        tb_ho = rem / P.Wo;
        tb_wo = rem - tb_ho * P.Wo;
    }
    auto fill_table = [&](int slot) {
        if (LINEAR) return;
        if (tid < BP) {
            unsigned off = kOutOfRange;
            if (tb_p < P.P) {
                int h = tb_ho * P.sh + oh, w = tb_wo * P.sw + ow;
                if ((unsigned)h < (unsigned)P.H && (unsigned)w < (unsigned)P.W)
                    off = (unsigned)((((tb_n * P.H + h) * P.W + w) * P.C) * 2);
            }
            xtab[slot * BP + tid] = off;
            tb_p += BP;
            tb_wo += adv_wo;
            int carry = tb_wo >= P.Wo;
            tb_wo -= carry ? P.Wo : 0;
            tb_ho += adv_ho + carry;
            carry = tb_ho >= P.Ho;
            tb_ho -= carry ? P.Ho : 0;
            tb_n += adv_n + carry;
        }
    };

    auto issue = [&](int step, int stage) {
        const int p0 = __builtin_amdgcn_readfirstlane((step0 + step) * BP);
        const unsigned sbase = (unsigned)__builtin_amdgcn_readfirstlane((int)(lds0 + stage * STAGE + fw * 1024));
        // dy: descriptor starts at pixel p0 and ends with the tensor
        const int4v rsrcG = make_rsrc(P.G + (long)p0 * P.K, (unsigned)((P.P - p0) * P.K) * 2u);
#pragma unroll
        for (int i = 0; i < PG; ++i) dma16(g_off[i], rsrcG, 0, sbase + i * RPG * BM * 2);
        if (LINEAR) {
            const int4v rsrcL = make_rsrc(P.X + (long)p0 * P.C, (unsigned)((P.P - p0) * P.C) * 2u);
#pragma unroll
            for (int i = 0; i < PX; ++i) dma16(x_add[i], rsrcL, 0, sbase + GBYTES + i * RPX * BN * 2);
        } else {
#pragma unroll
            for (int i = 0; i < PX; ++i) {
                unsigned xo = xtab[stage * BP + x_row[i]];
                unsigned voff = ((xo | x_add[i]) & kOutOfRange) ? kOutOfRange : xo + x_add[i];
                dma16(voff, rsrcX, 0, sbase + GBYTES + i * RPX * BN * 2);
            }
        }
    };

    typedef typename std::conditional<MF == 32, float16v, float4w>::type acc_t;
    acc_t acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c)
#pragma unroll
            for (int e = 0; e < ACCN; ++e) acc[a][c][e] = 0.f;

    auto compute = [&](int stage) {
        const unsigned char* sg = smem + stage * STAGE;
        const unsigned char* sx = sg + GBYTES;
#pragma unroll
        for (int kk = 0; kk < BP / KSTEP; ++kk) {
            half8 fa[FM], fb[FN];
#pragma unroll
            for (int a = 0; a < FM; ++a) {
                if (MF == 32) fa[a] = lds_frag_tr<BM>(sg, kk * 16, wm * WM + a * 32, lane);
                else fa[a] = lds_frag_tr_16<BM>(sg, kk * 32, wm * WM + a * 16, lane);
            }
#pragma unroll
            for (int c = 0; c < FN; ++c) {
                if (MF == 32) fb[c] = lds_frag_tr<BN>(sx, kk * 16, wn * WN + c * 32, lane);
                else fb[c] = lds_frag_tr_16<BN>(sx, kk * 32, wn * WN + c * 16, lane);
            }
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int c = 0; c < FN; ++c) {
                    if constexpr (MF == 32)
                        acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[a], fb[c], acc[a][c], 0, 0, 0);
                    else
                        acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa[a], fb[c], acc[a][c], 0, 0, 0);
                }
        }
    };

    // ---- ring pipeline ---------------------------------------------------------------------------
    if (nsteps > 0) {
#pragma unroll
        for (int q = 0; q < S; ++q)
            if (q < nsteps) fill_table(q);
        if (!LINEAR) __syncthreads();
        int issued = 0;
#pragma unroll
        for (int q = 0; q < S - 1; ++q)
            if (q < nsteps) { if (fetcher) issue(q, q); ++issued; }
        int cs = 0, is = (S - 1) % S;
        for (int it = 0; it < nsteps; ++it) {
            if (fetcher) { if (it + S - 2 < nsteps) wait_vmcnt<INFLIGHT>(); else wait_vmcnt<0>(); }
            if (!LINEAR) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // table writes landed
            __builtin_amdgcn_s_barrier();
            if (issued < nsteps) {
                if (fetcher) issue(issued, is);
                ++issued;
                is = (is + 1 == S) ? 0 : is + 1;
            }
            // table of step it+S (read by the issue of the next iteration) reuses the slot of
            // step `it`, whose loads were issued S-1 iterations ago
            if (it + S < nsteps) fill_table(cs);
            compute(cs);
            cs = (cs + 1 == S) ? 0 : cs + 1;
        }
    }

    // ---- store the fp32 tile: lanes 0..MF-1 hold consecutive channels of one filter row -----
    const long numel = (long)P.K * P.R * P.S * P.C;
    float* out = P.out + (long)split * numel;
    const int lcol = lane & (MF - 1), lhi = lane / MF;
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int c = 0; c < FN; ++c) {
            int col = c0 + wn * WN + c * MF + lcol;
            if (col >= P.C) continue;
#pragma unroll
            for (int e = 0; e < ACCN; ++e) {
                int k = (MF == 32) ? k0 + wm * WM + a * 32 + 8 * (e >> 2) + 4 * lhi + (e & 3)
                                   : k0 + wm * WM + a * 16 + 4 * lhi + e;
                if (k < P.K) out[((long)k * P.R * P.S + tap) * P.C + col] = acc[a][c][e];
            }
        }
}

template <int BM, int BN, int WGM, int WGN, int S, int BP, bool HF = false, int MF = 32>
static hipError_t launch_wdma(const WgradParams& P0, hipStream_t st)
{
    constexpr size_t lds = (size_t)S * BP * (BM + BN) * 2 + (size_t)S * BP * sizeof(unsigned);
    static_assert(lds <= 160 * 1024, "LDS budget");
    const bool linear = P0.R == 1 && P0.S == 1 && P0.sh == 1 && P0.sw == 1 && P0.ph == 0 && P0.pw == 0;
    static std::atomic<bool> configured{false};   // set once the attribute call has succeeded; a second thread may repeat it, harmlessly
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void*>(&wgrad_dma_kernel<BM, BN, WGM, WGN, S, BP, false, HF, MF>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(
            reinterpret_cast<const void*>(&wgrad_dma_kernel<BM, BN, WGM, WGN, S, BP, true, HF, MF>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    WgradParams P = P0;
    P.total_blocks = P.tiles_c * P.tiles_k * P.R * P.S * P.splits;
    const long blocks = ((long)P.total_blocks + 63) / 64 * 64;     // whole runs of 8 tiles on each of 8 XCDs
    if (linear)
        hipLaunchKernelGGL((wgrad_dma_kernel<BM, BN, WGM, WGN, S, BP, true, HF, MF>), dim3((unsigned)blocks),
                           dim3(64 * WGM * WGN), lds, st, P);
    else
        hipLaunchKernelGGL((wgrad_dma_kernel<BM, BN, WGM, WGN, S, BP, false, HF, MF>), dim3((unsigned)blocks),
                           dim3(64 * WGM * WGN), lds, st, P);
    return hipGetLastError();
}

const WgradVariant kWgradDmaVariants[kNumWgradDmaVariants] = {
    {128, 128, "wgrad_dma_128x128x64_4w_s2"},
    {128, 128, "wgrad_dma_128x128x32_4w_s3"},
    {256, 256, "wgrad_dma_256x256x64_8w_s2"},
    {256, 256, "wgrad_dma_256x256x32_8w_s3"},
    {64, 128, "wgrad_dma_64x128x64_4w_s3"},
    {256, 128, "wgrad_dma_256x128x32_8w_s3"},
    {64, 256, "wgrad_dma_64x256x64_4w_s2"},
    {64, 64, "wgrad_dma_64x64x64_4w_s3"},
    {128, 64, "wgrad_dma_128x64x64_4w_s3"},
    {256, 256, "wgrad_dma_256x256x64_8w_s2_hf"},
    {256, 256, "wgrad_dma_256x256x32_8w_s3_hf"},
    {256, 128, "wgrad_dma_256x128x32_8w_s3_hf"},
    {128, 128, "wgrad_dma_128x128x64_8w_s3_hf"},
    {256, 128, "wgrad_dma_256x128x64_8w_s3_hf"},
    {256, 256, "wgrad_dma_256x256x64_8w_s2_hf_m16"},
    {256, 256, "wgrad_dma_256x256x32_8w_s3_hf_m16"},
    {128, 128, "wgrad_dma_128x128x64_8w_s3_hf_m16"},
    {256, 128, "wgrad_dma_256x128x64_8w_s3_hf_m16"},
    {64, 64, "wgrad_dma_64x64x64_4w_s3_m16"},
    {128, 128, "wgrad_dma_128x128x64_4w_s2_m16"},
    {64, 128, "wgrad_dma_64x128x64_4w_s3_m16"},
};

hipError_t launch_wgrad_dma(int variant, const WgradParams& P, hipStream_t st)
{
    switch (variant) {
        case 0: return launch_wdma<128, 128, 2, 2, 2, 64>(P, st);
        case 1: return launch_wdma<128, 128, 2, 2, 3, 32>(P, st);
        case 2: return launch_wdma<256, 256, 2, 4, 2, 64>(P, st);
        case 3: return launch_wdma<256, 256, 2, 4, 3, 32>(P, st);
        case 4: return launch_wdma<64, 128, 1, 4, 3, 64>(P, st);
        case 5: return launch_wdma<256, 128, 4, 2, 3, 32>(P, st);
        case 6: return launch_wdma<64, 256, 1, 4, 2, 64>(P, st);
        case 7: return launch_wdma<64, 64, 2, 2, 3, 64>(P, st);
        case 8: return launch_wdma<128, 64, 2, 2, 3, 64>(P, st);
        case 9: return launch_wdma<256, 256, 2, 4, 2, 64, true>(P, st);
        case 10: return launch_wdma<256, 256, 2, 4, 3, 32, true>(P, st);
        case 11: return launch_wdma<256, 128, 4, 2, 3, 32, true>(P, st);
        case 12: return launch_wdma<128, 128, 2, 4, 3, 64, true>(P, st);
        case 13: return launch_wdma<256, 128, 4, 2, 3, 64, true>(P, st);
        case 14: return launch_wdma<256, 256, 2, 4, 2, 64, true, 16>(P, st);
        case 15: return launch_wdma<256, 256, 2, 4, 3, 32, true, 16>(P, st);
        case 16: return launch_wdma<128, 128, 2, 4, 3, 64, true, 16>(P, st);
        case 17: return launch_wdma<256, 128, 4, 2, 3, 64, true, 16>(P, st);
        case 18: return launch_wdma<64, 64, 2, 2, 3, 64, false, 16>(P, st);
        case 19: return launch_wdma<128, 128, 2, 2, 2, 64, false, 16>(P, st);
        case 20: return launch_wdma<64, 128, 1, 4, 3, 64, false, 16>(P, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sdconv
