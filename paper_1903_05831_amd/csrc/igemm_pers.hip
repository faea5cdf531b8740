// Persistent implicit-GEMM forward / data-gradient kernel.
//
// Same tiles, LDS layout, DMA addressing and MFMA mapping as igemm_dma.hip, but a workgroup
// does not end with its tile: a fixed grid (a few workgroups per compute unit) walks the tile
// list, and the load side of the ring runs ahead of the multiply side ACROSS tile borders.
// While the last contraction steps of one tile are multiplied and its result is converted and
// stored, the first steps of the next tile are already in flight, so the pipeline-fill
// latency, the tile set-up and the epilogue of the many short-contraction layers (1x1 convs
// with 64..256 channels: 2..8 steps per tile) overlap with useful work instead of adding up.
//
// The load side owns: the tile it fetches for, that tile's per-row offsets and tap masks, the
// (tap, channel-chunk) cursor.  The multiply side owns: its tile, the accumulators, the stage
// cursor.  They meet only in the ring: stage (n mod S) holds the n-th contraction step of the
// workgroup's whole tile sequence.
#include "common.h"
#include "igemm.h"
#include "dma.h"

namespace sdconv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));

struct TileInfo {
    int tn, cls, ca, cb, Hi, Wj, Mcls, m0, n0;
};

template <int MODE, int BM, int BN, int WGM, int WGN, int S, int BK>
__global__ __launch_bounds__(64 * WGM * WGN) void igemm_pers_kernel(IgemmParams P)
{
    constexpr int NW = WGM * WGN, NT = 64 * NW;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int CPR = BK / 8;
    constexpr int ROWB = BK * 2;
    constexpr int SWS = (CPR == 8) ? 1 : 2;
    constexpr int RPP = NT / CPR;
    constexpr int PA = BM / RPP, PB = BN / RPP;
    constexpr int STAGE = (BM + BN) * ROWB;
    constexpr int INFLIGHT = (S - 2) * (PA + PB);
    constexpr int kRun = 8;
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BM % RPP == 0 && BN % RPP == 0, "tile shape");
    static_assert(S >= 2 && INFLIGHT < 64, "pipeline depth");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
    // tap tables of every parity class: [class][tap] x {oh, ow, bo, ad}, then [class] counts
    const int RS = P.R * P.S;
    int* tap_oh = reinterpret_cast<int*>(smem + S * STAGE);
    int* tap_ow = tap_oh + P.nclasses * RS;
    int* tap_bo = tap_ow + P.nclasses * RS;
    int* tap_ad = tap_bo + P.nclasses * RS;
    int* tap_cnt = tap_ad + P.nclasses * RS;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, lhi = lane >> 5;

    if (wave == 0) {
        for (int cls = 0; cls < P.nclasses; ++cls) {
            const int ca = cls / P.sw_cls, cb = cls % P.sw_cls;
            bool ok = false;
            int oh = 0, ow = 0;
            const int r = lane / P.S, s = lane % P.S;
            if (lane < RS) {
                if (MODE == 0) { ok = true; oh = r * P.dh - P.ph; ow = s * P.dw - P.pw; }
                else {
                    int th = ca + P.ph - r * P.dh, tw = cb + P.pw - s * P.dw;
                    ok = (th % P.sh == 0) && (tw % P.sw == 0);
                    oh = th / P.sh; ow = tw / P.sw;
                }
            }
            unsigned long long mask = __ballot(ok);
            int pos = cls * RS + __popcll(mask & ((1ull << lane) - 1ull));
            if (ok) {
                tap_oh[pos] = oh; tap_ow[pos] = ow;
                tap_bo[pos] = (r * P.S + s) * P.Cs * 2;
                tap_ad[pos] = (oh * P.Ws + ow) * P.Cs * 2;
            }
            if (lane == 0) tap_cnt[cls] = __popcll(mask);
        }
    }
    __syncthreads();
    const int kchunks = (P.Cs + BK - 1) / BK;
    const int padded_tiles = ((P.total_tiles + 8 * kRun - 1) / (8 * kRun)) * (8 * kRun);

    // q-th entry of the chip-wide work list -> tile (runs of kRun consecutive tiles per XCD,
    // runs interleaved over the XCDs); false if the entry is padding
    auto tile_of = [&](int q, TileInfo& T) -> bool {
        const int xcd = q & 7, idx = q >> 3;
        const int tile = ((idx / kRun) * 8 + xcd) * kRun + (idx % kRun);
        if (tile >= P.total_tiles) return false;
        T.tn = tile % P.tiles_n;
        int tm = tile / P.tiles_n;
        int cls = 0;
        while (cls + 1 < P.nclasses && tm >= P.class_tile_start[cls + 1]) ++cls;
        tm -= P.class_tile_start[cls];
        T.cls = cls;
        T.ca = cls / P.sw_cls; T.cb = cls % P.sw_cls;
        if (MODE == 0) { T.Hi = P.Hd; T.Wj = P.Wd; }
        else { T.Hi = (P.Hd - T.ca + P.sh - 1) / P.sh; T.Wj = (P.Wd - T.cb + P.sw - 1) / P.sw; }
        T.Mcls = P.NB * T.Hi * T.Wj;
        T.m0 = tm * BM; T.n0 = T.tn * BN;
        return true;
    };

    // ---- load side -----------------------------------------------------------------------
    const int mh = (MODE == 0) ? P.sh : 1, mw = (MODE == 0) ? P.sw : 1;
    const int lrow = tid / CPR;
    const int kcl = (tid % CPR) ^ ((lrow >> SWS) & (CPR - 1));
    const int4v rsrcA = make_rsrc(P.A, (unsigned)(P.NB * P.Hs * P.Ws * P.Cs) * 2u);
    const int4v rsrcB = make_rsrc(P.B, (unsigned)(P.Cd * P.b_row_pitch) * 2u);
    unsigned a_off[PA];
    unsigned long long a_mask[PA];
    unsigned b_off[PB];
    int ld_q = (int)blockIdx.x - (int)gridDim.x;   // work-list cursor of the load side
    int ld_ntaps = 0, ld_tbase = 0, ld_tap = 0, ld_kc = 0;
    bool ld_live = false;                          // the load side still has steps to fetch

    // advance to the next tile that has contraction steps and prepare its row offsets
    auto ld_next_tile = [&]() {
        ld_live = false;
        for (;;) {
            ld_q += (int)gridDim.x;
            if (ld_q >= padded_tiles) return;
            TileInfo T;
            if (!tile_of(ld_q, T)) continue;
            const int nt = __builtin_amdgcn_readfirstlane(tap_cnt[T.cls]);
            if (nt == 0) continue;
            ld_ntaps = nt; ld_tbase = T.cls * RS; ld_tap = 0; ld_kc = 0;
#pragma unroll
            for (int p = 0; p < PA; ++p) {
                int m = T.m0 + lrow + RPP * p;
                a_off[p] = 0;
                a_mask[p] = 0ull;
                if (m < T.Mcls) {
                    int n = m / (T.Hi * T.Wj);
                    int rem = m - n * (T.Hi * T.Wj);
                    int i = rem / T.Wj, j = rem - i * T.Wj;
                    int ih = i * mh, jw = j * mw;
                    a_off[p] = (unsigned)((((n * P.Hs + ih) * P.Ws + jw) * P.Cs + kcl * 8) * 2);
                    unsigned long long mk = 0ull;
                    for (int t = 0; t < nt; ++t) {
                        int hs = ih + tap_oh[ld_tbase + t], ws = jw + tap_ow[ld_tbase + t];
                        if ((unsigned)hs < (unsigned)P.Hs && (unsigned)ws < (unsigned)P.Ws) mk |= 1ull << t;
                    }
                    a_mask[p] = mk;
                }
            }
#pragma unroll
            for (int p = 0; p < PB; ++p) {
                int n = T.n0 + lrow + RPP * p;
                b_off[p] = (n < P.Cd) ? (unsigned)((n * P.b_row_pitch + kcl * 8) * 2) : kOutOfRange;
            }
            ld_live = true;
            return;
        }
    };

    auto issue = [&](int stage) {
        const unsigned cbytes = (unsigned)__builtin_amdgcn_readfirstlane(ld_kc * ROWB);
        const unsigned cok = (ld_kc * BK + kcl * 8 < P.Cs) ? 1u : 0u;
        const unsigned ad = (unsigned)tap_ad[ld_tbase + ld_tap];
        const unsigned bo = (unsigned)__builtin_amdgcn_readfirstlane(tap_bo[ld_tbase + ld_tap]);
        const unsigned sbase = (unsigned)__builtin_amdgcn_readfirstlane((int)(lds0 + stage * STAGE + wave * 1024));
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            unsigned ok = cok & (unsigned)(a_mask[p] >> ld_tap);
            unsigned voff = (ok & 1u) ? a_off[p] + ad : kOutOfRange;
            dma16(voff, rsrcA, cbytes, sbase + p * RPP * ROWB);
        }
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            unsigned voff = cok ? b_off[p] : kOutOfRange;
            dma16(voff, rsrcB, bo + cbytes, sbase + BM * ROWB + p * RPP * ROWB);
        }
        // taps vary fastest (the taps of a 3x3 re-read nearly the same pixels back to back)
        int t1 = ld_tap + 1;
        bool wrap = t1 == ld_ntaps;
        ld_tap = __builtin_amdgcn_readfirstlane(wrap ? 0 : t1);
        ld_kc = __builtin_amdgcn_readfirstlane(wrap ? ld_kc + 1 : ld_kc);
        if (ld_kc == kchunks) ld_next_tile();
    };

    // ---- multiply side ---------------------------------------------------------------------
    float16v acc[FN][FM];
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

    // ---- fill the ring, then walk the tile list ------------------------------------------------
    int issued = 0, consumed = 0;       // contraction steps over the whole sequence
    int is = 0, cs = 0;                 // ring cursors
    ld_next_tile();
#pragma unroll
    for (int s = 0; s < S - 1; ++s)
        if (ld_live) { issue(is); ++issued; is = (is + 1 == S) ? 0 : is + 1; }

    for (int q = (int)blockIdx.x; q < padded_tiles; q += (int)gridDim.x) {
        TileInfo T;
        if (!tile_of(q, T)) continue;
        const int nk = __builtin_amdgcn_readfirstlane(tap_cnt[T.cls]) * kchunks;
#pragma unroll
        for (int a = 0; a < FN; ++a)
#pragma unroll
            for (int b = 0; b < FM; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

        for (int it = 0; it < nk; ++it) {
            // steps issued after the one about to be multiplied: allow them to stay in flight
            if (issued - consumed - 1 >= S - 2) wait_vmcnt<INFLIGHT>(); else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            if (ld_live) { issue(is); ++issued; is = (is + 1 == S) ? 0 : is + 1; }
            compute(cs);
            ++consumed;
            cs = (cs + 1 == S) ? 0 : cs + 1;
        }

        // epilogue: fp32 -> fp16 (nearest even), 8-byte NHWC stores
        const int eh = (MODE == 0) ? 1 : P.sh, ew = (MODE == 0) ? 1 : P.sw;
#pragma unroll
        for (int b = 0; b < FM; ++b) {
            int m = T.m0 + wm * WM + b * 32 + l32;
            if (m >= T.Mcls) continue;
            int n = m / (T.Hi * T.Wj);
            int rem = m - n * (T.Hi * T.Wj);
            int i = rem / T.Wj, j = rem - i * T.Wj;
            int hd = i * eh + T.ca, wd = j * ew + T.cb;
            __half* drow = P.D + ((n * P.Hd + hd) * P.Wd + wd) * P.Cd;
#pragma unroll
            for (int a = 0; a < FN; ++a) {
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    int col = T.n0 + wn * WN + a * 32 + 8 * qq + 4 * lhi;
                    if (col < P.Cd) {
                        half4 h;
                        h[0] = (_Float16)acc[a][b][4 * qq + 0];
                        h[1] = (_Float16)acc[a][b][4 * qq + 1];
                        h[2] = (_Float16)acc[a][b][4 * qq + 2];
                        h[3] = (_Float16)acc[a][b][4 * qq + 3];
                        *reinterpret_cast<half4*>(drow + col) = h;
                    }
                }
            }
        }
    }
}

static int device_cu_count()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
    }
    return cus;
}

template <int MODE, int BM, int BN, int WGM, int WGN, int S, int BK>
static hipError_t launch_pers_variant(const IgemmParams& P, hipStream_t st)
{
    const int RS = P.R * P.S;
    const size_t lds = (size_t)S * (BM + BN) * BK * 2 + (size_t)(4 * P.nclasses * RS + P.nclasses + 4) * sizeof(int);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    static bool configured = false;
    static int occ = 1;
    const void* fn = reinterpret_cast<const void*>(&igemm_pers_kernel<MODE, BM, BN, WGM, WGN, S, BK>);
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        int nb = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, 64 * WGM * WGN,
                                                         (size_t)S * (BM + BN) * BK * 2 + 1024);
        if (e != hipSuccess) return e;
        occ = nb < 1 ? 1 : nb;
        configured = true;
    }
    const int padded = ((P.total_tiles + 63) / 64) * 64;
    int grid = device_cu_count() * occ;
    grid = (grid / 8) * 8;
    if (grid > padded) grid = padded;
    if (grid < 8) grid = 8;
    hipLaunchKernelGGL((igemm_pers_kernel<MODE, BM, BN, WGM, WGN, S, BK>), dim3(grid), dim3(64 * WGM * WGN), lds, st, P);
    return hipGetLastError();
}

const IgemmVariant kIgemmPersVariants[kNumIgemmPersVariants] = {
    {128, 128, "igemm_fwd_pers_128x128x64_4w_s2", "igemm_dgrad_pers_128x128x64_4w_s2"},
    {128, 128, "igemm_fwd_pers_128x128x32_4w_s3", "igemm_dgrad_pers_128x128x32_4w_s3"},
    {128, 128, "igemm_fwd_pers_128x128x32_4w_s4", "igemm_dgrad_pers_128x128x32_4w_s4"},
    {256, 128, "igemm_fwd_pers_256x128x32_8w_s3", "igemm_dgrad_pers_256x128x32_8w_s3"},
    {128, 64, "igemm_fwd_pers_128x64x64_4w_s3", "igemm_dgrad_pers_128x64x64_4w_s3"},
    {128, 64, "igemm_fwd_pers_128x64x32_4w_s4", "igemm_dgrad_pers_128x64x32_4w_s4"},
    {256, 256, "igemm_fwd_pers_256x256x64_8w_s2", "igemm_dgrad_pers_256x256x64_8w_s2"},
    {256, 256, "igemm_fwd_pers_256x256x32_8w_s3", "igemm_dgrad_pers_256x256x32_8w_s3"},
    {256, 64, "igemm_fwd_pers_256x64x32_4w_s4", "igemm_dgrad_pers_256x64x32_4w_s4"},
    {128, 256, "igemm_fwd_pers_128x256x32_8w_s3", "igemm_dgrad_pers_128x256x32_8w_s3"},
};

#define SDCONV_PERS_CASE(idx, BM, BN, WGM, WGN, S, BK)                                         \
    case 2 * (idx): return launch_pers_variant<0, BM, BN, WGM, WGN, S, BK>(P, st);             \
    case 2 * (idx) + 1: return launch_pers_variant<1, BM, BN, WGM, WGN, S, BK>(P, st);

hipError_t launch_igemm_pers(int variant, const IgemmParams& P, hipStream_t st)
{
    const int key = variant * 2 + (P.mode ? 1 : 0);
    switch (key) {
        SDCONV_PERS_CASE(0, 128, 128, 2, 2, 2, 64)
        SDCONV_PERS_CASE(1, 128, 128, 2, 2, 3, 32)
        SDCONV_PERS_CASE(2, 128, 128, 2, 2, 4, 32)
        SDCONV_PERS_CASE(3, 256, 128, 4, 2, 3, 32)
        SDCONV_PERS_CASE(4, 128, 64, 2, 2, 3, 64)
        SDCONV_PERS_CASE(5, 128, 64, 2, 2, 4, 32)
        SDCONV_PERS_CASE(6, 256, 256, 2, 4, 2, 64)
        SDCONV_PERS_CASE(7, 256, 256, 2, 4, 3, 32)
        SDCONV_PERS_CASE(8, 256, 64, 4, 1, 4, 32)
        SDCONV_PERS_CASE(9, 128, 256, 2, 4, 3, 32)
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sdconv
