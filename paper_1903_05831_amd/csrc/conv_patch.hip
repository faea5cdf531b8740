// Stride-1 3x3-class forward / data-gradient kernel that keeps the input patch in LDS.
//
// The implicit-GEMM kernels fetch the activation tile once per filter tap: a 3x3 layer reads
// (nearly) the same pixels nine times from L2 and the global->LDS path, not the MFMA pipe,
// sets the pace.  Here a workgroup owns a TH x TW block of output pixels of one image and,
// per 64-channel slab, loads the (TH+2) x (TW+2) input patch ONCE (halo included, pixels
// outside the image zero-filled by the buffer range check = the padding).  The nine taps then
// read their A fragments from the same patch at a per-tap pixel displacement; only the filter
// slab (BN rows x 64 channels per tap) still streams through a ring, one stage per tap.
// Activation traffic drops from 9x to (TH+2)(TW+2)/(TH*TW) = 1.27x (16x16) per slab.
//
// Roles: either the upper half of the waves sends all loads (see igemm_ws.hip for why) and every
// wave multiplies, or extra waves do nothing but fetch (NDW below).  Two patch buffers alternate
// between slabs; the patch of slab kc+1 is requested at the first tap of slab kc and, because
// loads retire in order, has landed by the time the filter stage of its first tap has.
//
// Valid for stride 1, (R-1)*dil_h == 2 and (S-1)*dil_w == 2 (3x3 dilation 1 in particular),
// source channels a multiple of 64.  The data gradient of such a layer is the same kind of
// convolution over dy with displaced taps; it reads the filter as stored, [K][R][S][C], as
// 64-filter x BN-channel tiles that the transposing LDS read turns into fragments (lds_tr.h).
#include <type_traits>
#include "common.h"
#include "igemm.h"
#include "dma.h"
#include "igemm_epilogue.h"
#include "lds_tr.h"

namespace sdconv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4p __attribute__((ext_vector_type(4)));

// MF: 32 = v_mfma_f32_32x32x16_f16 blocks, 16 = v_mfma_f32_16x16x32_f16 blocks.
// NIW: number of fetching waves (the last NIW of the WGM x WGN waves); 0 = half of them.
// TH*TW need not be a multiple of the MFMA block height: the GEMM rows are padded up to
// WGM*MF and the padding rows are multiplied but never stored.  10 x 14 blocks tile the
// 100 x 168 and 50 x 84 feature maps of the res3 / res4 stages exactly (240 workgroups for
// 256 CUs with 128- resp. 64-wide filter tiles).
// TPS: taps per pipeline step (must divide R*S).  A step of one tap is only 64 deep; on small
// tiles the barrier and the wait then cost as much as the MFMAs between them, so a step can
// cover a whole filter row (TPS = 3): the ring stage holds TPS filter slabs.
// NPB: patch buffers.  Two alternate between channel slabs; a layer with 64 source channels has
// one slab and needs one buffer, which lets two or three workgroups share a compute unit's LDS
// (its 134 400-pixel maps make 546-1050 blocks: at one workgroup per unit they run in 3-4 rounds).
// NDW: waves that only fetch, beside the WGM x WGN multiplying ones (then none of those fetches).
// A wave stalls ~90 cycles in every LDS-DMA instruction it sends; with a dozen per step the
// fetching waves of a small block reach the barrier a thousand cycles after the others
// (timestamps of a 10 x 14 x 64 block: 1500 cycles of multiplying and 1200 of waiting per
// step).  Waves with nothing else to do take the stalls off that path.
template <int MODE, int TH, int TW, int BN, int WGM, int WGN, int SB, int MF = 32, int NIW = 0, int TPS = 1, int NPB = 2, int NDW = 0, bool TAIL = false>
__global__ __launch_bounds__(64 * (WGM * WGN + NDW)) void conv_patch_kernel(IgemmParams P)
{
    constexpr int EH = 2, EW = 2;                   // extra patch rows / columns
    constexpr int PH = TH + EH, PW = TW + EW, PPX = PH * PW;
    constexpr int NW = WGM * WGN, NI = NDW ? NDW : (NIW ? NIW : NW / 2), IW0 = NDW ? NW : NW - NI;
    constexpr int BM = TH * TW;                             // output pixels of the block
    constexpr int BMP = (BM + MF * WGM - 1) / (MF * WGM) * (MF * WGM);   // GEMM rows incl. padding
    constexpr int WM = BMP / WGM, WN = BN / WGN;
    constexpr int FM = WM / MF, FN = WN / MF;
    constexpr int ACCN = MF == 32 ? 16 : 4, KSTEP = MF == 32 ? 16 : 32, CPK = KSTEP / 8;
    constexpr int NPL = (PPX + 8 * NI - 1) / (8 * NI);     // patch loads per fetching lane
    constexpr int PATCHB = NPL * NI * 1024;                // bytes of one patch buffer
    constexpr int PB1 = BN / (8 * NI);                     // filter loads per fetching lane and tap
    constexpr int PB = TPS * PB1;                          // ... and step
    constexpr int BSLAB = BN * 128;                        // one tap's filter slab
    constexpr int BSTAGE = TPS * BSLAB;
    constexpr int D = SB - 1;                              // filter stages in flight
    static_assert((MF == 32 || MF == 16) && NI >= 1 && (NDW > 0 || NI < NW) && WM % MF == 0 && WN % MF == 0 && BN % (8 * NI) == 0, "tile shape");
    static_assert(SB >= 2 && NPL + D * PB < 64, "loads in flight");   // vmcnt is a 6-bit counter
    static_assert(NPB == 1 || NPB == 2, "patch buffers");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
    unsigned char* bring = smem + NPB * PATCHB;
    int* tap_bo = reinterpret_cast<int*>(bring + SB * BSTAGE);   // byte offset of the tap in a filter row
    int* tap_po = tap_bo + kMaxTaps;                              // patch-pixel displacement of the tap

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- which tile: runs of 8 consecutive tiles per XCD, runs interleaved over the XCDs ------
    constexpr int kRun = 8;
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int tile = ((idx / kRun) * 8 + xcd) * kRun + (idx % kRun);
    if (tile >= P.total_tiles) return;
    const int tn = tile % P.tiles_n;
    int t2 = tile / P.tiles_n;
    const int tx = t2 % P.tiles_w; t2 /= P.tiles_w;
    const int ty = t2 % P.tiles_h;
    const int n = t2 / P.tiles_h;
    const int h0 = ty * TH, w0 = tx * TW, n0 = tn * BN;

    // source pixel of output pixel (h, w) at tap (r, s): (h + oh, w + ow)
    const int oh_min = (MODE == 0) ? -P.ph : P.ph - (P.R - 1) * P.dh;
    const int ow_min = (MODE == 0) ? -P.pw : P.pw - (P.S - 1) * P.dw;
    const int ntaps = P.R * P.S;
    if (wave == 0 && lane < ntaps) {
        const int r = lane / P.S, s = lane % P.S;
        const int oh = (MODE == 0) ? r * P.dh - P.ph : P.ph - r * P.dh;
        const int ow = (MODE == 0) ? s * P.dw - P.pw : P.pw - s * P.dw;
        tap_bo[lane] = (r * P.S + s) * (MODE == 0 ? P.Cs : P.Cd) * 2;
        tap_po[lane] = (oh - oh_min) * PW + (ow - ow_min);
    }
    __syncthreads();
    const int kchunks = P.Cs / 64;
    const int ngroups = ntaps / TPS;                // steps per channel slab
    const int nk = ngroups * kchunks;

    // ---- fetching side ---------------------------------------------------------------------
    const bool fetcher = wave >= IW0;
    const int fw = wave - IW0;
    const int fpix = lane >> 3, fslot = lane & 7;   // pixel (or filter row) within an instruction, chunk slot
    unsigned a_off[NPL], b_off[PB1];
    if (fetcher) {
#pragma unroll
        for (int q = 0; q < NPL; ++q) {
            const int pp = (q * NI + fw) * 8 + fpix;            // patch pixel this lane fetches
            const int kcl = fslot ^ ((pp >> 1) & 7);            // logical chunk that lands in slot fslot
            const int pr = pp / PW, pc = pp - pr * PW;
            const int hs = h0 + oh_min + pr, ws = w0 + ow_min + pc;
            const bool ok = pp < PPX && (unsigned)hs < (unsigned)P.Hs && (unsigned)ws < (unsigned)P.Ws;
            a_off[q] = ok ? (unsigned)((((n * P.Hs + hs) * P.Ws + ws) * P.Cs + kcl * 8) * 2) : kOutOfRange;
        }
#pragma unroll
        for (int p = 0; p < PB1; ++p) {
            if (MODE == 0) {
                const int row = (p * NI + fw) * 8 + fpix;
                const int kcl = fslot ^ ((row >> 1) & 7);
                const int nn = n0 + row;
                b_off[p] = (nn < P.Cd) ? (unsigned)((nn * P.b_row_pitch + kcl * 8) * 2) : kOutOfRange;
            } else {
                // [64 filters][BN channels]: chunk slot (p*NI + fw)*64 + lane of the stage
                const int slot = (p * NI + fw) * 64 + lane;
                const int krow = slot / (BN / 8), pc = slot % (BN / 8);
                const int c = n0 + swizzled_chunk<BN>(krow, pc) * 8;
                b_off[p] = (c < P.Cd) ? (unsigned)((krow * P.b_row_pitch + c) * 2) : kOutOfRange;
            }
        }
    }
    const int4v rsrcA = make_rsrc(P.A, (unsigned)(P.NB * P.Hs * P.Ws * P.Cs) * 2u);
    const int4v rsrcB = make_rsrc(P.B, (unsigned)((MODE == 0 ? P.Cd : P.Cs) * P.b_row_pitch) * 2u);

    auto issue_patch = [&](int kc) {                // slab kc into buffer kc & 1
        const unsigned soff = (unsigned)__builtin_amdgcn_readfirstlane(kc * 128);
        const unsigned base = (unsigned)__builtin_amdgcn_readfirstlane((int)(lds0 + (kc & (NPB - 1)) * PATCHB + fw * 1024));
#pragma unroll
        for (int q = 0; q < NPL; ++q) dma16(a_off[q], rsrcA, soff, base + q * NI * 1024);
    };
    int nx_grp = 0, nx_kc = 0, nx_stage = 0;        // step the next issue_filter() fetches
    auto issue_filter = [&]() {
#pragma unroll
        for (int tt = 0; tt < TPS; ++tt) {
            const unsigned soff = (unsigned)__builtin_amdgcn_readfirstlane(
                tap_bo[nx_grp * TPS + tt] + (MODE == 0 ? nx_kc * 128 : nx_kc * 64 * P.b_row_pitch * 2));
            const unsigned base = (unsigned)__builtin_amdgcn_readfirstlane(
                (int)(lds0 + NPB * PATCHB + nx_stage * BSTAGE + tt * BSLAB + fw * 1024));
#pragma unroll
            for (int p = 0; p < PB1; ++p) dma16(b_off[p], rsrcB, soff, base + p * NI * 1024);
        }
        const int t1 = nx_grp + 1;
        const bool wrap = t1 == ngroups;
        nx_grp = __builtin_amdgcn_readfirstlane(wrap ? 0 : t1);
        nx_kc = __builtin_amdgcn_readfirstlane(wrap ? nx_kc + 1 : nx_kc);
        nx_stage = __builtin_amdgcn_readfirstlane(nx_stage + 1 == SB ? 0 : nx_stage + 1);
    };

    // ---- multiplying side ------------------------------------------------------------------
    const int wm = wave / WGN, wn = wave % WGN;
    const int frow = lane & (MF - 1), lhi = lane / MF;
    int pbase[FM];                                  // patch pixel of this lane's row at displacement 0
#pragma unroll
    for (int b = 0; b < FM; ++b) {
        const int ml = wm * WM + b * MF + frow;
        pbase[b] = (ml < BM) ? (ml / TW) * PW + (ml % TW) : 0;      // padding rows read pixel 0
    }
    typedef typename std::conditional<MF == 32, float16v, float4p>::type acc_t;
    acc_t acc[FN][FM];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int e = 0; e < ACCN; ++e) acc[a][b][e] = 0.f;

    auto compute = [&](int kc, int grp, int stage) {
        const unsigned char* pa = smem + (kc & (NPB - 1)) * PATCHB;
#pragma unroll
        for (int tt = 0; tt < TPS; ++tt) {
            const unsigned char* sb = bring + stage * BSTAGE + tt * BSLAB;
            const int po = __builtin_amdgcn_readfirstlane(tap_po[grp * TPS + tt]);
            int prow[FM];
#pragma unroll
            for (int b = 0; b < FM; ++b) prow[b] = pbase[b] + po;
#pragma unroll
            for (int kk = 0; kk < 64 / KSTEP; ++kk) {
                const int chunk = kk * CPK + lhi;
                half8 fa[FM], fb[FN];
#pragma unroll
                for (int b = 0; b < FM; ++b)
                    fa[b] = *reinterpret_cast<const half8*>(pa + prow[b] * 128 + ((chunk ^ ((prow[b] >> 1) & 7)) << 4));
#pragma unroll
                for (int a = 0; a < FN; ++a) {
                    if (MODE == 0) {
                        const int row = wn * WN + a * MF + frow;
                        fb[a] = *reinterpret_cast<const half8*>(sb + row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4));
                    } else if (MF == 32) {
                        fb[a] = lds_frag_tr<BN>(sb, kk * 16, wn * WN + a * 32, lane);
                    } else {
                        fb[a] = lds_frag_tr_16<BN>(sb, kk * 32, wn * WN + a * 16, lane);
                    }
                }
#pragma unroll
                for (int a = 0; a < FN; ++a)
#pragma unroll
                    for (int b = 0; b < FM; ++b) {
                        if constexpr (MF == 32)
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[a], fa[b], acc[a][b], 0, 0, 0);
                        else
                            acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fb[a], fa[b], acc[a][b], 0, 0, 0);
                    }
            }
        }
    };

    // ---- pipeline: one step per (slab, group of TPS taps), taps fastest ------------------------------------
    if (fetcher) {
        issue_patch(0);
#pragma unroll
        for (int s = 0; s < D; ++s)
            if (s < nk) issue_filter();
    }
    int tap = 0, kc = 0, stage = 0;
    for (int t = 0; t < nk; ++t) {
        // loads retire in order: once the filter stage of step t is in, so is everything sent
        // before it, in particular the patch of its slab (sent at least ntaps - D steps earlier)
        // (the next slab's patch, sent at tap 0 between two filter stages, may stay in flight
        // while it is younger than the stage awaited here)
        if (fetcher) {
            const bool patch_younger = tap >= 1 && tap <= D - 1 && kc + 1 < kchunks;
            if (t + D - 1 >= nk) wait_vmcnt<0>();
            else if (patch_younger) wait_vmcnt<(D - 1) * PB + NPL>();
            else wait_vmcnt<(D - 1) * PB>();
        }
        __builtin_amdgcn_s_barrier();
        if (fetcher) {
            if (tap == 0 && kc + 1 < kchunks) issue_patch(kc + 1);   // its buffer was last read in slab kc-1
            if (t + D < nk) issue_filter();
        }
        if (NDW == 0 || wave < NW) compute(kc, tap, stage);
        stage = (stage + 1 == SB) ? 0 : stage + 1;
        if (++tap == ngroups) { tap = 0; ++kc; }
    }

    // ---- epilogue ------------------------------------------------------------------------------
    static_assert(NW * epilogue_strip_bytes<WN, MF>() <= NPB * PATCHB + SB * TPS * BN * 128,
                  "epilogue strips fit in the patch buffers and the filter ring");
    __builtin_amdgcn_s_barrier();                   // everybody is done reading the last patch and filter stage
    if (NDW > 0 && wave >= NW) return;              // no barrier follows
    store_rows_via_lds<FM, FN, MF, TAIL>(acc, smem + wave * epilogue_strip_bytes<WN, MF>(), lane, n0 + wn * WN, P,
                               [&](int r) -> long {
        const int ml = wm * WM + r;
        const int h = h0 + ml / TW, w = w0 + ml % TW;
        if (ml >= BM || h >= P.Hd || w >= P.Wd) return -1;
        return ((long)n * P.Hd + h) * P.Wd + w;
    });
}

template <int MODE, int TH, int TW, int BN, int WGM, int WGN, int SB, int MF = 32, int NIW = 0, int TPS = 1, int NPB = 2, int NDW = 0, bool TAIL>
static hipError_t launch_patch_variant_impl(const IgemmParams& P, hipStream_t st)
{
    if ((P.R * P.S) % TPS != 0 || (P.R * P.S) / TPS < SB - 1) return hipErrorInvalidValue;
    if (NPB == 1 && P.Cs != 64) return hipErrorInvalidValue;      // one patch buffer = one channel slab
    constexpr int NI = NDW ? NDW : (NIW ? NIW : WGM * WGN / 2);
    constexpr int NPL = ((TH + 2) * (TW + 2) + 8 * NI - 1) / (8 * NI);
    constexpr size_t lds = (size_t)NPB * NPL * NI * 1024 + (size_t)SB * TPS * BN * 128 + 2 * kMaxTaps * sizeof(int);
    static_assert(lds <= 160 * 1024, "LDS budget");
    static std::atomic<bool> configured{false};   // set once the attribute call has succeeded; a second thread may repeat it, harmlessly
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void*>(&conv_patch_kernel<MODE, TH, TW, BN, WGM, WGN, SB, MF, NIW, TPS, NPB, NDW, TAIL>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    const int grid = ((P.total_tiles + 63) / 64) * 64;
    hipLaunchKernelGGL((conv_patch_kernel<MODE, TH, TW, BN, WGM, WGN, SB, MF, NIW, TPS, NPB, NDW, TAIL>), dim3(grid), dim3(64 * (WGM * WGN + NDW)),
                       lds, st, P);
    return hipGetLastError();
}

template <int MODE, int TH, int TW, int BN, int WGM, int WGN, int SB, int MF = 32, int NIW = 0, int TPS = 1, int NPB = 2, int NDW = 0>
static hipError_t launch_patch_variant(const IgemmParams& P, hipStream_t st)
{
    // the tail has kernels of its own: see store_rows_via_lds
    return P.ep.any() ? launch_patch_variant_impl<MODE, TH, TW, BN, WGM, WGN, SB, MF, NIW, TPS, NPB, NDW, true>(P, st) : launch_patch_variant_impl<MODE, TH, TW, BN, WGM, WGN, SB, MF, NIW, TPS, NPB, NDW, false>(P, st);
}

const PatchVariant kPatchVariants[kNumPatchVariants] = {
    {16, 16, 128, 1, 3, "conv_fwd_patch_16x16x128_s3", "conv_dgrad_patch_16x16x128_s3"},
    {8, 16, 128, 1, 4, "conv_fwd_patch_8x16x128_s4", "conv_dgrad_patch_8x16x128_s4"},
    {8, 16, 256, 1, 3, "conv_fwd_patch_8x16x256_s3", "conv_dgrad_patch_8x16x256_s3"},
    {16, 16, 64, 1, 4, "conv_fwd_patch_16x16x64_s4", "conv_dgrad_patch_16x16x64_s4"},
    {8, 32, 128, 1, 3, "conv_fwd_patch_8x32x128_s3", "conv_dgrad_patch_8x32x128_s3"},
    {8, 16, 64, 1, 4, "conv_fwd_patch_8x16x64_s4", "conv_dgrad_patch_8x16x64_s4"},
    {16, 16, 128, 1, 3, "conv_fwd_patch_16x16x128_s3_m16", "conv_dgrad_patch_16x16x128_s3_m16"},
    {8, 16, 128, 1, 4, "conv_fwd_patch_8x16x128_s4_m16", "conv_dgrad_patch_8x16x128_s4_m16"},
    {16, 16, 64, 1, 4, "conv_fwd_patch_16x16x64_s4_m16", "conv_dgrad_patch_16x16x64_s4_m16"},
    {8, 32, 128, 1, 3, "conv_fwd_patch_8x32x128_s3_m16", "conv_dgrad_patch_8x32x128_s3_m16"},
    {10, 14, 128, 1, 4, "conv_fwd_patch_10x14x128_6w_s4_m16", "conv_dgrad_patch_10x14x128_6w_s4_m16"},
    {10, 14, 64, 1, 4, "conv_fwd_patch_10x14x64_6w_s4_m16", "conv_dgrad_patch_10x14x64_6w_s4_m16"},
    {10, 14, 128, 1, 4, "conv_fwd_patch_10x14x128_12w_s4_m16", "conv_dgrad_patch_10x14x128_12w_s4_m16"},
    {10, 14, 64, 1, 4, "conv_fwd_patch_10x14x64_6w1f_s4_m16", "conv_dgrad_patch_10x14x64_6w1f_s4_m16"},
    {10, 14, 64, 3, 3, "conv_fwd_patch_10x14x64_6w_s3_m16_t3", "conv_dgrad_patch_10x14x64_6w_s3_m16_t3"},
    {10, 14, 128, 3, 2, "conv_fwd_patch_10x14x128_12w_s2_m16_t3", "conv_dgrad_patch_10x14x128_12w_s2_m16_t3"},
    {10, 14, 128, 3, 2, "conv_fwd_patch_10x14x128_6w_s2_m16_t3", "conv_dgrad_patch_10x14x128_6w_s2_m16_t3"},
    {16, 16, 64, 3, 2, "conv_fwd_patch_16x16x64_s2_m16_t3", "conv_dgrad_patch_16x16x64_s2_m16_t3"},
    {10, 14, 64, 3, 3, "conv_fwd_patch_10x14x64_12w_s3_m16_t3", "conv_dgrad_patch_10x14x64_12w_s3_m16_t3"},
    {10, 14, 64, 3, 4, "conv_fwd_patch_10x14x64_6w_s4_m16_t3", "conv_dgrad_patch_10x14x64_6w_s4_m16_t3"},
    {16, 16, 64, 3, 3, "conv_fwd_patch_16x16x64_s3_m16_t3_2f", "conv_dgrad_patch_16x16x64_s3_m16_t3_2f"},
    {8, 16, 128, 3, 2, "conv_fwd_patch_8x16x128_s2_m16_t3", "conv_dgrad_patch_8x16x128_s2_m16_t3"},
    // one patch buffer: layers with 64 source channels only
    {16, 16, 64, 1, 3, "conv_fwd_patch_16x16x64_s3_m16_1p", "conv_dgrad_patch_16x16x64_s3_m16_1p", 1},
    {16, 16, 64, 3, 2, "conv_fwd_patch_16x16x64_s2_m16_t3_1p", "conv_dgrad_patch_16x16x64_s2_m16_t3_1p", 1},
    {10, 14, 64, 1, 3, "conv_fwd_patch_10x14x64_6w_s3_m16_1p", "conv_dgrad_patch_10x14x64_6w_s3_m16_1p", 1},
    {10, 14, 64, 3, 2, "conv_fwd_patch_10x14x64_6w_s2_m16_t3_1p", "conv_dgrad_patch_10x14x64_6w_s2_m16_t3_1p", 1},
    {8, 16, 64, 1, 3, "conv_fwd_patch_8x16x64_s3_m16_1p", "conv_dgrad_patch_8x16x64_s3_m16_1p", 1},
    {8, 16, 64, 3, 2, "conv_fwd_patch_8x16x64_s2_m16_t3_1p", "conv_dgrad_patch_8x16x64_s2_m16_t3_1p", 1},
    // waves that only fetch beside the multiplying ones
    {10, 14, 64, 3, 4, "conv_fwd_patch_10x14x64_6w2f_s4_m16_t3", "conv_dgrad_patch_10x14x64_6w2f_s4_m16_t3"},
    {10, 14, 64, 3, 3, "conv_fwd_patch_10x14x64_6w2f_s3_m16_t3", "conv_dgrad_patch_10x14x64_6w2f_s3_m16_t3"},
    {10, 14, 128, 3, 2, "conv_fwd_patch_10x14x128_12w4f_s2_m16_t3", "conv_dgrad_patch_10x14x128_12w4f_s2_m16_t3"},
    {10, 14, 128, 3, 2, "conv_fwd_patch_10x14x128_6w2f_s2_m16_t3", "conv_dgrad_patch_10x14x128_6w2f_s2_m16_t3"},
    {16, 16, 64, 3, 2, "conv_fwd_patch_16x16x64_8w2f_s2_m16_t3", "conv_dgrad_patch_16x16x64_8w2f_s2_m16_t3"},
    {10, 14, 64, 3, 2, "conv_fwd_patch_10x14x64_6w2f_s2_m16_t3_1p", "conv_dgrad_patch_10x14x64_6w2f_s2_m16_t3_1p", 1},
    {10, 14, 64, 1, 3, "conv_fwd_patch_10x14x64_6w2f_s3_m16_1p", "conv_dgrad_patch_10x14x64_6w2f_s3_m16_1p", 1},
    {10, 14, 64, 3, 4, "conv_fwd_patch_10x14x64_6w4f_s4_m16_t3", "conv_dgrad_patch_10x14x64_6w4f_s4_m16_t3"},
};

#define SDCONV_PATCH_CASE(idx, TH, TW, BN, WGM, WGN, SB)                                      \
    case 2 * (idx): return launch_patch_variant<0, TH, TW, BN, WGM, WGN, SB>(P, st);          \
    case 2 * (idx) + 1: return launch_patch_variant<1, TH, TW, BN, WGM, WGN, SB>(P, st);

hipError_t launch_conv_patch(int variant, const IgemmParams& P, hipStream_t st)
{
    const int key = variant * 2 + (P.mode ? 1 : 0);
    switch (key) {
        SDCONV_PATCH_CASE(0, 16, 16, 128, 4, 2, 3)
        SDCONV_PATCH_CASE(1, 8, 16, 128, 2, 4, 4)
        SDCONV_PATCH_CASE(2, 8, 16, 256, 2, 4, 3)
        SDCONV_PATCH_CASE(3, 16, 16, 64, 4, 2, 4)
        SDCONV_PATCH_CASE(4, 8, 32, 128, 4, 2, 3)
        SDCONV_PATCH_CASE(5, 8, 16, 64, 4, 2, 4)
        case 12: return launch_patch_variant<0, 16, 16, 128, 4, 2, 3, 16>(P, st);
        case 13: return launch_patch_variant<1, 16, 16, 128, 4, 2, 3, 16>(P, st);
        case 14: return launch_patch_variant<0, 8, 16, 128, 2, 4, 4, 16>(P, st);
        case 15: return launch_patch_variant<1, 8, 16, 128, 2, 4, 4, 16>(P, st);
        case 16: return launch_patch_variant<0, 16, 16, 64, 4, 2, 4, 16>(P, st);
        case 17: return launch_patch_variant<1, 16, 16, 64, 4, 2, 4, 16>(P, st);
        case 18: return launch_patch_variant<0, 8, 32, 128, 4, 2, 3, 16>(P, st);
        case 19: return launch_patch_variant<1, 8, 32, 128, 4, 2, 3, 16>(P, st);
        case 20: return launch_patch_variant<0, 10, 14, 128, 3, 2, 4, 16, 2>(P, st);
        case 21: return launch_patch_variant<1, 10, 14, 128, 3, 2, 4, 16, 2>(P, st);
        case 22: return launch_patch_variant<0, 10, 14, 64, 3, 2, 4, 16, 2>(P, st);
        case 23: return launch_patch_variant<1, 10, 14, 64, 3, 2, 4, 16, 2>(P, st);
        case 24: return launch_patch_variant<0, 10, 14, 128, 3, 4, 4, 16, 4>(P, st);
        case 25: return launch_patch_variant<1, 10, 14, 128, 3, 4, 4, 16, 4>(P, st);
        case 26: return launch_patch_variant<0, 10, 14, 64, 3, 2, 4, 16, 1>(P, st);
        case 27: return launch_patch_variant<1, 10, 14, 64, 3, 2, 4, 16, 1>(P, st);
        case 28: return launch_patch_variant<0, 10, 14, 64, 3, 2, 3, 16, 2, 3>(P, st);
        case 29: return launch_patch_variant<1, 10, 14, 64, 3, 2, 3, 16, 2, 3>(P, st);
        case 30: return launch_patch_variant<0, 10, 14, 128, 3, 4, 2, 16, 4, 3>(P, st);
        case 31: return launch_patch_variant<1, 10, 14, 128, 3, 4, 2, 16, 4, 3>(P, st);
        case 32: return launch_patch_variant<0, 10, 14, 128, 3, 2, 2, 16, 2, 3>(P, st);
        case 33: return launch_patch_variant<1, 10, 14, 128, 3, 2, 2, 16, 2, 3>(P, st);
        case 34: return launch_patch_variant<0, 16, 16, 64, 4, 2, 2, 16, 0, 3>(P, st);
        case 35: return launch_patch_variant<1, 16, 16, 64, 4, 2, 2, 16, 0, 3>(P, st);
        case 36: return launch_patch_variant<0, 10, 14, 64, 3, 4, 3, 16, 4, 3>(P, st);
        case 37: return launch_patch_variant<1, 10, 14, 64, 3, 4, 3, 16, 4, 3>(P, st);
        case 38: return launch_patch_variant<0, 10, 14, 64, 3, 2, 4, 16, 2, 3>(P, st);
        case 39: return launch_patch_variant<1, 10, 14, 64, 3, 2, 4, 16, 2, 3>(P, st);
        case 40: return launch_patch_variant<0, 16, 16, 64, 4, 2, 3, 16, 2, 3>(P, st);
        case 41: return launch_patch_variant<1, 16, 16, 64, 4, 2, 3, 16, 2, 3>(P, st);
        case 42: return launch_patch_variant<0, 8, 16, 128, 2, 4, 2, 16, 0, 3>(P, st);
        case 43: return launch_patch_variant<1, 8, 16, 128, 2, 4, 2, 16, 0, 3>(P, st);
        case 44: return launch_patch_variant<0, 16, 16, 64, 4, 2, 3, 16, 0, 1, 1>(P, st);
        case 45: return launch_patch_variant<1, 16, 16, 64, 4, 2, 3, 16, 0, 1, 1>(P, st);
        case 46: return launch_patch_variant<0, 16, 16, 64, 4, 2, 2, 16, 0, 3, 1>(P, st);
        case 47: return launch_patch_variant<1, 16, 16, 64, 4, 2, 2, 16, 0, 3, 1>(P, st);
        case 48: return launch_patch_variant<0, 10, 14, 64, 3, 2, 3, 16, 2, 1, 1>(P, st);
        case 49: return launch_patch_variant<1, 10, 14, 64, 3, 2, 3, 16, 2, 1, 1>(P, st);
        case 50: return launch_patch_variant<0, 10, 14, 64, 3, 2, 2, 16, 2, 3, 1>(P, st);
        case 51: return launch_patch_variant<1, 10, 14, 64, 3, 2, 2, 16, 2, 3, 1>(P, st);
        case 52: return launch_patch_variant<0, 8, 16, 64, 4, 2, 3, 16, 0, 1, 1>(P, st);
        case 53: return launch_patch_variant<1, 8, 16, 64, 4, 2, 3, 16, 0, 1, 1>(P, st);
        case 54: return launch_patch_variant<0, 8, 16, 64, 4, 2, 2, 16, 0, 3, 1>(P, st);
        case 55: return launch_patch_variant<1, 8, 16, 64, 4, 2, 2, 16, 0, 3, 1>(P, st);
        case 56: return launch_patch_variant<0, 10, 14, 64, 3, 2, 4, 16, 0, 3, 2, 2>(P, st);
        case 57: return launch_patch_variant<1, 10, 14, 64, 3, 2, 4, 16, 0, 3, 2, 2>(P, st);
        case 58: return launch_patch_variant<0, 10, 14, 64, 3, 2, 3, 16, 0, 3, 2, 2>(P, st);
        case 59: return launch_patch_variant<1, 10, 14, 64, 3, 2, 3, 16, 0, 3, 2, 2>(P, st);
        case 60: return launch_patch_variant<0, 10, 14, 128, 3, 4, 2, 16, 0, 3, 2, 4>(P, st);
        case 61: return launch_patch_variant<1, 10, 14, 128, 3, 4, 2, 16, 0, 3, 2, 4>(P, st);
        case 62: return launch_patch_variant<0, 10, 14, 128, 3, 2, 2, 16, 0, 3, 2, 2>(P, st);
        case 63: return launch_patch_variant<1, 10, 14, 128, 3, 2, 2, 16, 0, 3, 2, 2>(P, st);
        case 64: return launch_patch_variant<0, 16, 16, 64, 4, 2, 2, 16, 0, 3, 2, 2>(P, st);
        case 65: return launch_patch_variant<1, 16, 16, 64, 4, 2, 2, 16, 0, 3, 2, 2>(P, st);
        case 66: return launch_patch_variant<0, 10, 14, 64, 3, 2, 2, 16, 0, 3, 1, 2>(P, st);
        case 67: return launch_patch_variant<1, 10, 14, 64, 3, 2, 2, 16, 0, 3, 1, 2>(P, st);
        case 68: return launch_patch_variant<0, 10, 14, 64, 3, 2, 3, 16, 0, 1, 1, 2>(P, st);
        case 69: return launch_patch_variant<1, 10, 14, 64, 3, 2, 3, 16, 0, 1, 1, 2>(P, st);
        case 70: return launch_patch_variant<0, 10, 14, 64, 3, 2, 4, 16, 0, 3, 2, 4>(P, st);
        case 71: return launch_patch_variant<1, 10, 14, 64, 3, 2, 4, 16, 0, 3, 2, 4>(P, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sdconv
