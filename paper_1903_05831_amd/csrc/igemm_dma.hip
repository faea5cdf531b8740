// Implicit-GEMM forward / data-gradient kernel with an asynchronous global->LDS pipeline.
//
// Same mathematics and tile decomposition as igemm.hip (rows = pixels gathered on the fly,
// columns = filters, contraction over taps x channels in steps of 64 halves), but the tiles
// travel HBM/L2 -> LDS with buffer_load_dwordx4 ... lds (no VGPR staging, no ds_write) into a
// ring of S stages, so S-1 contraction steps are in flight while one is multiplied.
//
// The DMA instruction writes LDS at M0 + lane*16: one wave instruction fills 8 rows of
// 128 bytes.  The 16-byte chunks of a row are XOR-swizzled with (row>>1)&7 so that the MFMA
// fragment reads (16 consecutive rows, one chunk column) touch all 64 banks once; the
// swizzle is applied on the global side by choosing which chunk a lane fetches.
//
// Addressing is kept off the vector ALU: each lane holds one byte offset per tile row (its
// pixel at tap (0,0)) and a bit mask saying which taps fall inside the image for that row;
// per contraction step a load costs one add (the uniform tap displacement) and one select.
// Lanes whose tap is outside the image, or whose row is past the tile edge, get an offset
// beyond the buffer descriptor's range: the hardware range check then writes zeros to LDS
// and never touches memory.  The channel-chunk offset rides in the scalar offset operand.
//
// The loads are issued through inline assembly and retired with explicit
// s_waitcnt vmcnt(n): the compiler's own wait insertion treats every LDS-DMA as aliasing all
// of LDS and would drain the whole ring before each fragment read.
#include "common.h"
#include "igemm.h"
#include "dma.h"
#include "igemm_epilogue.h"

namespace sdconv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));

// BK = contraction halves per stage (64 or 32): a tile row is BK*2 bytes = CPR 16-byte chunks.
// Dynamic LDS of a variant: the ring and the tap tables, or the epilogue strips if those need more.
template <int BM, int BN, int WGM, int WGN, int S, int BK> constexpr size_t dma_lds_bytes()
{
    constexpr size_t loop = (size_t)S * (BM + BN) * BK * 2 + (4 * kMaxTaps + 4) * sizeof(int);
    constexpr size_t strips = (size_t)WGM * WGN * epilogue_strip_bytes<BN / WGN>();
    return loop > strips ? loop : strips;
}

template <int MODE, int BM, int BN, int WGM, int WGN, int S, int BK, bool TAIL = false>
__global__ __launch_bounds__(64 * WGM * WGN) void igemm_dma_kernel(IgemmParams P)
{
    constexpr int NW = WGM * WGN, NT = 64 * NW;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int CPR = BK / 8;                     // 16-byte chunks per tile row
    constexpr int ROWB = BK * 2;                    // bytes per tile row
    constexpr int SWS = (CPR == 8) ? 1 : 2;         // swizzle: chunk ^= (row >> SWS) & (CPR-1)
    constexpr int RPP = NT / CPR;                   // tile rows one pass of all threads covers
    constexpr int PA = BM / RPP, PB = BN / RPP;     // DMA loads per thread and stage
    constexpr int STAGE = (BM + BN) * ROWB;         // bytes
    constexpr int INFLIGHT = (S - 2) * (PA + PB);   // loads that may stay outstanding
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BM % RPP == 0 && BN % RPP == 0, "tile shape");
    static_assert(S >= 2 && INFLIGHT < 64, "pipeline depth");
    static_assert(BK == 64 || BK == 32, "contraction step");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
    int* tap_oh = reinterpret_cast<int*>(smem + S * STAGE);
    int* tap_ow = tap_oh + kMaxTaps;
    int* tap_bo = tap_ow + kMaxTaps;      // byte offset of the tap inside a filter row
    int* tap_ad = tap_bo + kMaxTaps;      // byte displacement of the tap in the source image
    int* tap_cnt = tap_ad + kMaxTaps;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    // ---- which tile: workgroups go round-robin over the 8 XCDs; hand each XCD runs of kRun
    // consecutive tiles (shared rows and halos meet in one L2) and interleave the runs, so
    // that cheap and expensive parity classes of a strided dgrad spread over all XCDs ----
    constexpr int kRun = 8;
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int tile = ((idx / kRun) * 8 + xcd) * kRun + (idx % kRun);
    if (tile >= P.total_tiles) return;
    const int tn = tile % P.tiles_n;
    int tm = tile / P.tiles_n;
    int cls = 0;
    while (cls + 1 < P.nclasses && tm >= P.class_tile_start[cls + 1]) ++cls;
    tm -= P.class_tile_start[cls];
    const int ca = cls / P.sw_cls, cb = cls % P.sw_cls;

    int Hi, Wj, mh, mw, eh, ew;
    if (MODE == 0) { Hi = P.Hd; Wj = P.Wd; mh = P.sh; mw = P.sw; eh = 1; ew = 1; }
    else {
        Hi = (P.Hd - ca + P.sh - 1) / P.sh; Wj = (P.Wd - cb + P.sw - 1) / P.sw;
        mh = 1; mw = 1; eh = P.sh; ew = P.sw;
    }
    const int Mcls = P.NB * Hi * Wj;
    const int m0 = tm * BM, n0 = tn * BN;

    // ---- tap table -------------------------------------------------------------------
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
        if (ok) {
            tap_oh[pos] = oh; tap_ow[pos] = ow;
            tap_bo[pos] = (r * P.S + s) * P.Cs * 2;
            tap_ad[pos] = (oh * P.Ws + ow) * P.Cs * 2;
        }
        if (lane == 0) tap_cnt[0] = __popcll(mask);
    }
    __syncthreads();
    const int ntaps = __builtin_amdgcn_readfirstlane(tap_cnt[0]);
    const int kchunks = (P.Cs + BK - 1) / BK;
    const int nk = ntaps * kchunks;

    // ---- per-thread DMA rows -------------------------------------------------------------
    const int lrow = tid / CPR;                                         // 0 .. RPP-1
    const int kcl = (tid % CPR) ^ ((lrow >> SWS) & (CPR - 1));          // logical 16-byte chunk this lane fetches
    unsigned a_off[PA];                 // byte offset of the row's pixel at tap displacement 0
    unsigned long long a_mask[PA];      // bit t: tap t of this row lies inside the source image
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        int m = m0 + lrow + RPP * p;
        a_off[p] = 0;
        a_mask[p] = 0ull;
        if (m < Mcls) {
            int n = m / (Hi * Wj);
            int rem = m - n * (Hi * Wj);
            int i = rem / Wj, j = rem - i * Wj;
            int ih = i * mh, jw = j * mw;
            a_off[p] = (unsigned)((((n * P.Hs + ih) * P.Ws + jw) * P.Cs + kcl * 8) * 2);
            unsigned long long mk = 0ull;
            for (int t = 0; t < ntaps; ++t) {
                int hs = ih + tap_oh[t], ws = jw + tap_ow[t];
                if ((unsigned)hs < (unsigned)P.Hs && (unsigned)ws < (unsigned)P.Ws) mk |= 1ull << t;
            }
            a_mask[p] = mk;
        }
    }
    unsigned b_off[PB];
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        int n = n0 + lrow + RPP * p;
        b_off[p] = (n < P.Cd) ? (unsigned)((n * P.b_row_pitch + kcl * 8) * 2) : kOutOfRange;
    }
    const int4v rsrcA = make_rsrc(P.A, (unsigned)(P.NB * P.Hs * P.Ws * P.Cs) * 2u);
    const int4v rsrcB = make_rsrc(P.B, (unsigned)(P.Cd * P.b_row_pitch) * 2u);

    int nx_tap = 0, nx_kc = 0;          // contraction step the next issue() fetches (wave-uniform)
    auto issue = [&](int stage) {
        const unsigned cbytes = (unsigned)nx_kc * (unsigned)ROWB;
        const unsigned cok = (nx_kc * BK + kcl * 8 < P.Cs) ? 1u : 0u;
        const unsigned ad = (unsigned)tap_ad[nx_tap];
        const unsigned bo = (unsigned)__builtin_amdgcn_readfirstlane(tap_bo[nx_tap]);
        const unsigned sbase = lds0 + stage * STAGE + wave * 1024;
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            unsigned ok = cok & (unsigned)(a_mask[p] >> nx_tap);
            unsigned voff = (ok & 1u) ? a_off[p] + ad : kOutOfRange;
            dma16(voff, rsrcA, cbytes, sbase + p * RPP * ROWB);
        }
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            unsigned voff = cok ? b_off[p] : kOutOfRange;
            dma16(voff, rsrcB, bo + cbytes, sbase + BM * ROWB + p * RPP * ROWB);
        }
        // taps vary fastest: the 9 taps of a 3x3 re-read nearly the same pixels of one
        // 64-channel slab back to back, while it is still in L2
        int t1 = nx_tap + 1;
        bool wrap = t1 == ntaps;
        nx_tap = __builtin_amdgcn_readfirstlane(wrap ? 0 : t1);
        nx_kc = __builtin_amdgcn_readfirstlane(wrap ? nx_kc + 1 : nx_kc);
    };

    float16v acc[FN][FM];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

    const int l32 = lane & 31, lhi = lane >> 5;
    auto compute = [&](int stage) {
        const unsigned char* sa = smem + stage * STAGE;
        const unsigned char* sb = sa + BM * ROWB;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int chunk = kk * 2 + lhi;
            half8 fa[FM], fb[FN];
#pragma unroll
            for (int b = 0; b < FM; ++b) {
                int row = wm * WM + b * 32 + l32;
                fa[b] = *reinterpret_cast<const half8*>(sa + row * ROWB + ((chunk ^ ((row >> SWS) & (CPR - 1))) << 4));
            }
#pragma unroll
            for (int a = 0; a < FN; ++a) {
                int row = wn * WN + a * 32 + l32;
                fb[a] = *reinterpret_cast<const half8*>(sb + row * ROWB + ((chunk ^ ((row >> SWS) & (CPR - 1))) << 4));
            }
#pragma unroll
            for (int a = 0; a < FN; ++a)
#pragma unroll
                for (int b = 0; b < FM; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[a], fa[b], acc[a][b], 0, 0, 0);
        }
    };

    // ---- ring pipeline: S-1 steps in flight ---------------------------------------------------
    {
        int issued = 0;
#pragma unroll
        for (int s = 0; s < S - 1; ++s)
            if (s < nk) { issue(s); ++issued; }
        int cs = 0;                 // stage being multiplied
        int is = (S - 1) % S;       // stage the next issue() fills
        for (int it = 0; it < nk; ++it) {
            if (it + S - 2 < nk) wait_vmcnt<INFLIGHT>(); else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            if (issued < nk) { issue(is); ++issued; is = (is + 1 == S) ? 0 : is + 1; }
            compute(cs);
            cs = (cs + 1 == S) ? 0 : cs + 1;
        }
    }

    // ---- epilogue: through a per-wave LDS strip into 16-byte NHWC stores --------------------
    // (the strips may run over the tap tables behind the ring: those are dead by now)
    static_assert(NW * epilogue_strip_bytes<WN>() <= dma_lds_bytes<BM, BN, WGM, WGN, S, BK>(), "epilogue strips fit in LDS");
    __builtin_amdgcn_s_barrier();                   // everybody is done reading the last stage
    store_tile_via_lds<FM, FN, 32, TAIL>(acc, smem + wave * epilogue_strip_bytes<WN>(), lane, m0 + wm * WM, n0 + wn * WN,
                               Mcls, P, Hi, Wj, eh, ew, ca, cb);
}

template <int MODE, int BM, int BN, int WGM, int WGN, int S, int BK, bool TAIL>
static hipError_t launch_dma_variant_impl(const IgemmParams& P, hipStream_t st)
{
    constexpr size_t lds = dma_lds_bytes<BM, BN, WGM, WGN, S, BK>();
    static_assert(lds <= 160 * 1024, "LDS budget");
    static std::atomic<bool> configured{false};   // set once the attribute call has succeeded; a second thread may repeat it, harmlessly
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void*>(&igemm_dma_kernel<MODE, BM, BN, WGM, WGN, S, BK, TAIL>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    const int grid = ((P.total_tiles + 63) / 64) * 64;   // whole runs of 8 tiles on each of 8 XCDs
    hipLaunchKernelGGL((igemm_dma_kernel<MODE, BM, BN, WGM, WGN, S, BK, TAIL>), dim3(grid), dim3(64 * WGM * WGN), lds, st, P);
    return hipGetLastError();
}

template <int MODE, int BM, int BN, int WGM, int WGN, int S, int BK>
static hipError_t launch_dma_variant(const IgemmParams& P, hipStream_t st)
{
    // the tail has kernels of its own: see store_rows_via_lds
    return P.ep.any() ? launch_dma_variant_impl<MODE, BM, BN, WGM, WGN, S, BK, true>(P, st) : launch_dma_variant_impl<MODE, BM, BN, WGM, WGN, S, BK, false>(P, st);
}

const IgemmVariant kIgemmDmaVariants[kNumIgemmDmaVariants] = {
    {128, 128, "igemm_fwd_dma_128x128x64_4w_s2", "igemm_dgrad_dma_128x128x64_4w_s2"},
    {128, 128, "igemm_fwd_dma_128x128x32_4w_s3", "igemm_dgrad_dma_128x128x32_4w_s3"},
    {128, 128, "igemm_fwd_dma_128x128x32_4w_s4", "igemm_dgrad_dma_128x128x32_4w_s4"},
    {128, 128, "igemm_fwd_dma_128x128x32_4w_s5", "igemm_dgrad_dma_128x128x32_4w_s5"},
    {256, 128, "igemm_fwd_dma_256x128x64_8w_s3", "igemm_dgrad_dma_256x128x64_8w_s3"},
    {256, 128, "igemm_fwd_dma_256x128x32_8w_s3", "igemm_dgrad_dma_256x128x32_8w_s3"},
    {128, 64, "igemm_fwd_dma_128x64x64_4w_s3", "igemm_dgrad_dma_128x64x64_4w_s3"},
    {128, 64, "igemm_fwd_dma_128x64x32_4w_s4", "igemm_dgrad_dma_128x64x32_4w_s4"},
    {256, 256, "igemm_fwd_dma_256x256x64_8w_s2", "igemm_dgrad_dma_256x256x64_8w_s2"},
    {256, 256, "igemm_fwd_dma_256x256x32_8w_s3", "igemm_dgrad_dma_256x256x32_8w_s3"},
    {256, 256, "igemm_fwd_dma_256x256x32_8w_s4", "igemm_dgrad_dma_256x256x32_8w_s4"},
    {256, 256, "igemm_fwd_dma_256x256x32_8w_s4_w64x128", "igemm_dgrad_dma_256x256x32_8w_s4_w64x128"},
    // shallower rings of the 128x64 tile: more workgroups per compute unit for the HBM-bound
    // 1x1 layers of res2, whose contraction is two to eight steps long
    {128, 64, "igemm_fwd_dma_128x64x32_4w_s2", "igemm_dgrad_dma_128x64x32_4w_s2"},
    {128, 64, "igemm_fwd_dma_128x64x32_4w_s3", "igemm_dgrad_dma_128x64x32_4w_s3"},
};

#define SDCONV_DMA_CASE(idx, BM, BN, WGM, WGN, S, BK)                                         \
    case 2 * (idx): return launch_dma_variant<0, BM, BN, WGM, WGN, S, BK>(P, st);             \
    case 2 * (idx) + 1: return launch_dma_variant<1, BM, BN, WGM, WGN, S, BK>(P, st);

hipError_t launch_igemm_dma(int variant, const IgemmParams& P, hipStream_t st)
{
    const int key = variant * 2 + (P.mode ? 1 : 0);
    switch (key) {
        SDCONV_DMA_CASE(0, 128, 128, 2, 2, 2, 64)
        SDCONV_DMA_CASE(1, 128, 128, 2, 2, 3, 32)
        SDCONV_DMA_CASE(2, 128, 128, 2, 2, 4, 32)
        SDCONV_DMA_CASE(3, 128, 128, 2, 2, 5, 32)
        SDCONV_DMA_CASE(4, 256, 128, 4, 2, 3, 64)
        SDCONV_DMA_CASE(5, 256, 128, 4, 2, 3, 32)
        SDCONV_DMA_CASE(6, 128, 64, 2, 2, 3, 64)
        SDCONV_DMA_CASE(7, 128, 64, 2, 2, 4, 32)
        SDCONV_DMA_CASE(8, 256, 256, 2, 4, 2, 64)
        SDCONV_DMA_CASE(9, 256, 256, 2, 4, 3, 32)
        SDCONV_DMA_CASE(10, 256, 256, 2, 4, 4, 32)
        SDCONV_DMA_CASE(11, 256, 256, 4, 2, 4, 32)
        SDCONV_DMA_CASE(12, 128, 64, 2, 2, 2, 32)
        SDCONV_DMA_CASE(13, 128, 64, 2, 2, 3, 32)
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sdconv
