// Implicit-GEMM forward / data-gradient kernel with separate fetching and multiplying waves.
//
// Same tiles, LDS layout, swizzle and contraction order as igemm_dma.hip.  What differs is who
// sends the global->LDS loads.  A wave that issues buffer_load ... lds stalls until the texture
// path has taken the instruction (about 16-20 cycles per 1 KiB instruction, per CU), and while
// it stalls it cannot feed the matrix pipe.  When every wave fetches and then multiplies, all
// waves of a SIMD stall together and the fetch time adds to the MFMA time.  Here
//   NP > 0 : NP extra waves do nothing but fetch (they own no part of the tile), the WGM x WGN
//            multiplying waves never touch global memory until the epilogue;
//   NP == 0: the upper half of the multiplying waves fetches for everybody.  With two waves per
//            SIMD (wave w and w + NWC/2 share one) the lower wave multiplies while the upper one
//            is stalled in its burst of loads, then the upper one multiplies.
// One workgroup barrier per contraction step, shared by both kinds of wave, orders the ring.
//
// The data gradient (MODE 1) reads the filter as it is stored, [K][R][S][C]: its B tile is 64
// filters (contraction rows) x BN input channels, kept in LDS in that orientation and turned
// into fragments by the transposing LDS read (lds_tr.h), so no transposed copy of the filter
// is needed.  The forward pass keeps the [row][64 contraction halves] tiles of igemm_dma.hip.
//
// Row addressing is computed once per workgroup by all threads (one tile row each: byte offset
// of the pixel at tap displacement 0 and a bit mask of the taps inside the image) and handed to
// the fetching waves through LDS.
#include <type_traits>
#include "common.h"
#include "igemm.h"
#include "dma.h"
#include "igemm_epilogue.h"
#include "lds_tr.h"

namespace sdconv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v_ __attribute__((ext_vector_type(4)));

// MF: 32 = v_mfma_f32_32x32x16_f16 blocks; 16 = v_mfma_f32_16x16x32_f16 blocks, for tile heights
// that are a multiple of 16 but not of 32 per wave row (224 = 2 x 112 rows: 25088 = 112 x 224
// pixels of the RoI head then give 224 or 896 tiles instead of 196 or 784 for 256 CUs).
// The work of one workgroup on tile `tile` of a launch (or of a part of one, see
// igemm_ws_mixed_kernel) with `tiles_n` column tiles whose row tiles start at row tile `tm0`.
template <int MODE, int BM, int BN, int WGM, int WGN, int S, int BK, int NP, int MF = 32, bool TAIL = false>
__device__ __forceinline__ void igemm_ws_body(const IgemmParams& P, const int tile, const int tiles_n, const int tm0)
{
    constexpr int NWC = WGM * WGN;                  // multiplying waves
    constexpr int NW = NWC + NP, NT = 64 * NW;
    constexpr int NI = NP ? NP : NWC / 2;           // fetching waves
    constexpr int IW0 = NP ? NWC : NWC / 2;         // first fetching wave
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / MF, FN = WN / MF;
    constexpr int ACCN = MF == 32 ? 16 : 4;         // accumulator floats per lane and block
    constexpr int CPR = BK / 8;                     // 16-byte chunks per tile row
    constexpr int ROWB = BK * 2;                    // bytes per tile row
    constexpr int SWS = (CPR == 8) ? 1 : 2;         // swizzle: chunk ^= (row >> SWS) & (CPR-1)
    constexpr int RPP = 64 * NI / CPR;              // tile rows one pass of the fetching waves covers
    constexpr int PA = BM / RPP, PB = BN / RPP;     // loads per fetching thread and stage
    constexpr int STAGE = (BM + BN) * ROWB;         // bytes
    constexpr int INFLIGHT = (S - 2) * (PA + PB);   // loads a fetching wave may leave outstanding
    static_assert((MF == 32 || MF == 16) && WM % MF == 0 && WN % MF == 0 && BM % RPP == 0 && BN % RPP == 0, "tile shape");
    static_assert(MF == 32 || BK == 64, "16x16x32 blocks take 32 contraction values per instruction");
    static_assert(S >= 2 && INFLIGHT < 64, "pipeline depth");
    static_assert(BK == 64 || BK == 32, "contraction step");
    static_assert(MODE == 0 || (BK == 64 && (64 * NI) % (BN / 8) == 0), "data-gradient filter tile");
    static_assert(NI >= 1 && (NP > 0 || NWC % 2 == 0), "fetching waves");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
    int* tap_oh = reinterpret_cast<int*>(smem + S * STAGE);
    int* tap_ow = tap_oh + kMaxTaps;
    int* tap_bo = tap_ow + kMaxTaps;      // byte offset of the tap inside a filter row
    int* tap_ad = tap_bo + kMaxTaps;      // byte displacement of the tap in the source image
    int* tap_cnt = tap_ad + kMaxTaps;     // [4]
    unsigned* row_off = reinterpret_cast<unsigned*>(tap_cnt + 4);                    // [BM]
    unsigned long long* row_mask = reinterpret_cast<unsigned long long*>(row_off + BM);   // [BM]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int tn = tile % tiles_n;
    int tm = tile / tiles_n + tm0;
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
            tap_bo[pos] = (r * P.S + s) * (MODE == 0 ? P.Cs : P.Cd) * 2;
            tap_ad[pos] = (oh * P.Ws + ow) * P.Cs * 2;
        }
        if (lane == 0) tap_cnt[0] = __popcll(mask);
    }
    __syncthreads();
    const int ntaps = __builtin_amdgcn_readfirstlane(tap_cnt[0]);
    if (MODE == 1 && !TAIL && ntaps == 0) {
        // a class without taps (three of the four of a 1x1 stride-2 layer): nothing to multiply
        if (wave < NWC)
            store_zero_subtile<WM, WN>(lane, m0 + (wave / WGN) * WM, n0 + (wave % WGN) * WN, Mcls, P, Hi, Wj, eh, ew, ca, cb);
        return;
    }
    const int kchunks = (P.Cs + BK - 1) / BK;
    const int nk = ntaps * kchunks;

    // ---- row table: one tile row per thread ------------------------------------------------
    for (int r = tid; r < BM; r += NT) {
        int m = m0 + r;
        unsigned off = 0;
        unsigned long long mk = 0ull;
        if (m < Mcls) {
            int n = m / (Hi * Wj);
            int rem = m - n * (Hi * Wj);
            int i = rem / Wj, j = rem - i * Wj;
            int ih = i * mh, jw = j * mw;
            off = (unsigned)((((n * P.Hs + ih) * P.Ws + jw) * P.Cs) * 2);
            for (int t = 0; t < ntaps; ++t) {
                int hs = ih + tap_oh[t], ws = jw + tap_ow[t];
                if ((unsigned)hs < (unsigned)P.Hs && (unsigned)ws < (unsigned)P.Ws) mk |= 1ull << t;
            }
        }
        row_off[r] = off;
        row_mask[r] = mk;
    }
    __syncthreads();

    const bool fetcher = wave >= IW0;

    // ---- fetching side ---------------------------------------------------------------------
    const int ft = tid - IW0 * 64;                  // thread index among the fetching threads
    const int fw = wave - IW0;                      // fetching wave index
    const int lrow = ft / CPR;                      // 0 .. RPP-1 (fetching threads only)
    const int kc = ft % CPR;                        // 16-byte chunk slot in LDS this lane fills
    unsigned a_off[PA];
    unsigned long long a_mask[PA];
    unsigned b_off[PB];
    int b_krow[PB];                                 // MODE 1: filter (contraction row) of each load
    const bool partial = (P.Cs % BK) != 0;          // last channel chunk is short
    if (fetcher) {
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            const int r = lrow + RPP * p;
            const int kcl = kc ^ ((r >> SWS) & (CPR - 1));      // logical chunk this lane fetches
            a_off[p] = row_off[r] + (unsigned)(kcl * 16);
            a_mask[p] = row_mask[r];
        }
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            if (MODE == 0) {
                const int r = lrow + RPP * p;
                const int kcl = kc ^ ((r >> SWS) & (CPR - 1));
                const int n = n0 + r;
                b_off[p] = (n < P.Cd) ? (unsigned)((n * P.b_row_pitch + kcl * 8) * 2) : kOutOfRange;
            } else {
                // [64 filters][BN channels]: chunk slot (p*64*NI + ft) of the stage
                const int slot = p * 64 * NI + ft;
                const int krow = slot / (BN / 8), pc = slot % (BN / 8);
                const int c = n0 + swizzled_chunk<BN>(krow, pc) * 8;
                b_krow[p] = krow;
                b_off[p] = (c < P.Cd) ? (unsigned)((krow * P.b_row_pitch + c) * 2) : kOutOfRange;
            }
        }
    }
    const int4v rsrcA = make_rsrc(P.A, (unsigned)(P.NB * P.Hs * P.Ws * P.Cs) * 2u);
    const int4v rsrcB = make_rsrc(P.B, (unsigned)((MODE == 0 ? P.Cd : P.Cs) * P.b_row_pitch) * 2u);

    int nx_tap = 0, nx_kc = 0;          // contraction step the next issue() fetches (wave-uniform)
    auto issue = [&](int stage) {
        const unsigned cbytes = (unsigned)__builtin_amdgcn_readfirstlane(nx_kc * ROWB);
        const unsigned ad = (unsigned)tap_ad[nx_tap];
        const unsigned bo = (unsigned)__builtin_amdgcn_readfirstlane(tap_bo[nx_tap]);
        const unsigned sbase = (unsigned)__builtin_amdgcn_readfirstlane((int)(lds0 + stage * STAGE + fw * 1024));
        const int cleft = P.Cs - nx_kc * BK;        // channels left from this chunk's start
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            const int r = lrow + RPP * p;
            const int kcl = kc ^ ((r >> SWS) & (CPR - 1));
            unsigned ok = (unsigned)(a_mask[p] >> nx_tap) & 1u;
            if (partial && kcl * 8 >= cleft) ok = 0;
            unsigned voff = ok ? a_off[p] + ad : kOutOfRange;
            dma16(voff, rsrcA, cbytes, sbase + p * RPP * ROWB);
        }
        if (MODE == 0) {
#pragma unroll
            for (int p = 0; p < PB; ++p) {
                const int r = lrow + RPP * p;
                const int kcl = kc ^ ((r >> SWS) & (CPR - 1));
                unsigned voff = (partial && kcl * 8 >= cleft) ? kOutOfRange : b_off[p];
                dma16(voff, rsrcB, bo + cbytes, sbase + BM * ROWB + p * RPP * ROWB);
            }
        } else {
            // filters nx_kc*64 .. +63 of tap nx_tap, BN channels each
            const unsigned kbytes = (unsigned)__builtin_amdgcn_readfirstlane(nx_kc * BK * P.b_row_pitch * 2);
#pragma unroll
            for (int p = 0; p < PB; ++p) {
                unsigned voff = (partial && b_krow[p] >= cleft) ? kOutOfRange : b_off[p];
                dma16(voff, rsrcB, bo + kbytes, sbase + BM * ROWB + p * NI * 1024);
            }
        }
        // taps vary fastest: the taps of a 3x3 re-read nearly the same pixels of one channel
        // slab back to back, while it is still in L2
        int t1 = nx_tap + 1;
        bool wrap = t1 == ntaps;
        nx_tap = __builtin_amdgcn_readfirstlane(wrap ? 0 : t1);
        nx_kc = __builtin_amdgcn_readfirstlane(wrap ? nx_kc + 1 : nx_kc);
    };

    if (NP > 0 && fetcher) {
        // ---- dedicated fetching wave: S-1 steps ahead of the multipliers ---------------------
#pragma unroll
        for (int s = 0; s < S - 1; ++s)
            if (s < nk) issue(s);
        int is = (S - 1) % S;
        for (int it = 0; it < nk; ++it) {
            if (it + S - 2 < nk) wait_vmcnt<INFLIGHT>(); else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();           // step it is in LDS; stage of step it-1 is free
            if (it + S - 1 < nk) { issue(is); is = (is + 1 == S) ? 0 : is + 1; }
        }
        return;
    }

    // ---- multiplying side ------------------------------------------------------------------
    const int wm = wave / WGN, wn = wave % WGN;
    typedef typename std::conditional<MF == 32, float16v, float4v_>::type acc_t;
    acc_t acc[FN][FM];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int e = 0; e < ACCN; ++e) acc[a][b][e] = 0.f;

    // fragment lane mapping: row (or column) lane % MF of a block, contraction chunk lane / MF
    const int frow = lane & (MF - 1), lhi = lane / MF;
    constexpr int KSTEP = MF == 32 ? 16 : 32;       // contraction values per MFMA
    constexpr int CPK = KSTEP / 8;                  // 16-byte chunks per MFMA step
    auto compute = [&](int stage) {
        const unsigned char* sa = smem + stage * STAGE;
        const unsigned char* sb = sa + BM * ROWB;
#pragma unroll
        for (int kk = 0; kk < BK / KSTEP; ++kk) {
            const int chunk = kk * CPK + lhi;
            half8 fa[FM], fb[FN];
#pragma unroll
            for (int b = 0; b < FM; ++b) {
                int row = wm * WM + b * MF + frow;
                fa[b] = *reinterpret_cast<const half8*>(sa + row * ROWB + ((chunk ^ ((row >> SWS) & (CPR - 1))) << 4));
            }
#pragma unroll
            for (int a = 0; a < FN; ++a) {
                if (MODE == 0) {
                    int row = wn * WN + a * MF + frow;
                    fb[a] = *reinterpret_cast<const half8*>(sb + row * ROWB + ((chunk ^ ((row >> SWS) & (CPR - 1))) << 4));
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
    };

    if (NP > 0) {
        int cs = 0;
        for (int it = 0; it < nk; ++it) {
            __builtin_amdgcn_s_barrier();
            compute(cs);
            cs = (cs + 1 == S) ? 0 : cs + 1;
        }
    } else {
        // upper half of the waves fetches for the whole group, then multiplies its own share
        if (fetcher) {
#pragma unroll
            for (int s = 0; s < S - 1; ++s)
                if (s < nk) issue(s);
        }
        int cs = 0, is = (S - 1) % S;
        for (int it = 0; it < nk; ++it) {
            if (fetcher) { if (it + S - 2 < nk) wait_vmcnt<INFLIGHT>(); else wait_vmcnt<0>(); }
            __builtin_amdgcn_s_barrier();
            if (fetcher && it + S - 1 < nk) issue(is);
            is = (is + 1 == S) ? 0 : is + 1;
            compute(cs);
            cs = (cs + 1 == S) ? 0 : cs + 1;
        }
    }

    // ---- epilogue: through a per-wave LDS strip into 16-byte NHWC stores --------------------
    static_assert(NWC * epilogue_strip_bytes<WN, MF>() <= S * STAGE, "epilogue strips fit in the ring");
    __builtin_amdgcn_s_barrier();                   // everybody is done reading the last stage
    store_tile_via_lds<FM, FN, MF, TAIL>(acc, smem + wave * epilogue_strip_bytes<WN, MF>(), lane, m0 + wm * WM, n0 + wn * WN,
                               Mcls, P, Hi, Wj, eh, ew, ca, cb);
}

// Which tile a workgroup takes: runs of kRun consecutive tiles per XCD (workgroup b runs on XCD
// b % 8), runs interleaved over the XCDs.  Consecutive tiles are the column tiles of one row
// tile, which read the same activation rows: a run keeps them on one L2.  Measured on the
// detector step: runs of 2 beat runs of 1 (every L2 fetches every activation row), and runs of
// 4, 8 and 16 (fewer row tiles per XCD in flight at a time), by 0.5-0.9 %.
__device__ __forceinline__ int xcd_run_tile(int b)
{
    constexpr int kRun = 2;
    const int xcd = b & 7, idx = b >> 3;
    return ((idx / kRun) * 8 + xcd) * kRun + (idx % kRun);
}

template <int MODE, int BM, int BN, int WGM, int WGN, int S, int BK, int NP, int MF = 32, bool TAIL = false>
__global__ __launch_bounds__(64 * (WGM * WGN + NP)) void igemm_ws_kernel(IgemmParams P)
{
    const int tile = xcd_run_tile(blockIdx.x);
    if (tile >= P.total_tiles) return;
    igemm_ws_body<MODE, BM, BN, WGM, WGN, S, BK, NP, MF, TAIL>(P, tile, P.tiles_n, 0);
}

// Two tile widths in one launch.  A layer whose tiles make a few whole rounds of the chip's
// compute units plus half a round (896 tiles of 224 x 256 on 256 CUs: the 1x1 layers of the RoI
// head) leaves half the units idle for the last round.  Here the first mix_big_tiles tiles are
// BN wide and the row tiles after them are cut into tiles of half the width, twice as many and
// ~0.64 of the time each, so the last round fills the chip.  Undivided images only (one parity
// class); both bodies have the same waves.
template <int MODE, int BM, int BN, int BNS, int WGM, int WGN, int S, int SS, int BK, int MF, bool TAIL>
__global__ __launch_bounds__(64 * WGM * WGN) void igemm_ws_mixed_kernel(IgemmParams P)
{
    int b = blockIdx.x;
    if (b < P.mix_big_blocks) {
        const int tile = xcd_run_tile(b);
        if (tile >= P.mix_big_tiles) return;
        igemm_ws_body<MODE, BM, BN, WGM, WGN, S, BK, 0, MF, TAIL>(P, tile, P.tiles_n, 0);
    } else {
        const int tile = xcd_run_tile(b - P.mix_big_blocks);
        if (tile >= P.mix_small_tiles) return;
        igemm_ws_body<MODE, BM, BNS, WGM, WGN, SS, BK, 0, MF, TAIL>(P, tile, P.mix_small_tiles_n, P.mix_small_tm0);
    }
}

template <int MODE, int BM, int BN, int BNS, int WGM, int WGN, int S, int SS, int BK, int MF, bool TAIL>
static hipError_t launch_ws_mixed_impl(const IgemmParams& P0, hipStream_t st)
{
    constexpr size_t lds_big = (size_t)S * (BM + BN) * BK * 2, lds_small = (size_t)SS * (BM + BNS) * BK * 2;
    constexpr size_t lds = (lds_big > lds_small ? lds_big : lds_small) + (4 * kMaxTaps + 4) * sizeof(int) + (size_t)BM * 12;
    static_assert(lds <= 160 * 1024, "LDS budget");
    if (P0.nclasses != 1) return hipErrorInvalidValue;
    static std::atomic<bool> configured{false};   // set once the attribute call has succeeded; a second thread may repeat it, harmlessly
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void*>(&igemm_ws_mixed_kernel<MODE, BM, BN, BNS, WGM, WGN, S, SS, BK, MF, TAIL>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    // P0.tiles_n / P0.total_tiles describe the launch in BN-wide tiles.  Whole rounds of 256
    // workgroups stay BN wide (rounded down to whole row tiles); the rest is cut in two.
    IgemmParams P = P0;
    const int row_tiles = P0.total_tiles / P0.tiles_n;
    int big_rows = (P0.total_tiles / 256 * 256) / P0.tiles_n;
    if (2 * (P0.total_tiles % 256) > 256 + P0.tiles_n) big_rows = row_tiles;     // the half tiles would need two rounds
    P.mix_big_tiles = big_rows * P0.tiles_n;
    P.mix_big_blocks = (P.mix_big_tiles + 63) / 64 * 64;
    P.mix_small_tm0 = big_rows;
    P.mix_small_tiles_n = (P0.Cd + BNS - 1) / BNS;
    P.mix_small_tiles = (row_tiles - big_rows) * P.mix_small_tiles_n;
    const int grid = P.mix_big_blocks + (P.mix_small_tiles + 63) / 64 * 64;
    if (grid == 0) return hipSuccess;
    hipLaunchKernelGGL((igemm_ws_mixed_kernel<MODE, BM, BN, BNS, WGM, WGN, S, SS, BK, MF, TAIL>), dim3(grid),
                       dim3(64 * WGM * WGN), lds, st, P);
    return hipGetLastError();
}

template <int MODE, int BM, int BN, int BNS, int WGM, int WGN, int S, int SS, int BK, int MF>
static hipError_t launch_ws_mixed(const IgemmParams& P, hipStream_t st)
{
    return P.ep.any() ? launch_ws_mixed_impl<MODE, BM, BN, BNS, WGM, WGN, S, SS, BK, MF, true>(P, st)
                      : launch_ws_mixed_impl<MODE, BM, BN, BNS, WGM, WGN, S, SS, BK, MF, false>(P, st);
}

template <int MODE, int BM, int BN, int WGM, int WGN, int S, int BK, int NP, int MF = 32, bool TAIL>
static hipError_t launch_ws_variant_impl(const IgemmParams& P, hipStream_t st)
{
    constexpr size_t lds = (size_t)S * (BM + BN) * BK * 2 + (4 * kMaxTaps + 4) * sizeof(int) + (size_t)BM * 12;
    static_assert(lds <= 160 * 1024, "LDS budget");
    static std::atomic<bool> configured{false};   // set once the attribute call has succeeded; a second thread may repeat it, harmlessly
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void*>(&igemm_ws_kernel<MODE, BM, BN, WGM, WGN, S, BK, NP, MF, TAIL>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    const int grid = ((P.total_tiles + 63) / 64) * 64;   // whole runs of tiles on each of 8 XCDs
    hipLaunchKernelGGL((igemm_ws_kernel<MODE, BM, BN, WGM, WGN, S, BK, NP, MF, TAIL>), dim3(grid),
                       dim3(64 * (WGM * WGN + NP)), lds, st, P);
    return hipGetLastError();
}

template <int MODE, int BM, int BN, int WGM, int WGN, int S, int BK, int NP, int MF = 32>
static hipError_t launch_ws_variant(const IgemmParams& P, hipStream_t st)
{
    // the tail has kernels of its own: see store_rows_via_lds
    return P.ep.any() ? launch_ws_variant_impl<MODE, BM, BN, WGM, WGN, S, BK, NP, MF, true>(P, st) : launch_ws_variant_impl<MODE, BM, BN, WGM, WGN, S, BK, NP, MF, false>(P, st);
}

const IgemmVariant kIgemmWsVariants[kNumIgemmWsVariants] = {
    {128, 128, "igemm_fwd_ws_128x128x64_4w2f_s3", "igemm_dgrad_ws_128x128x64_4w2f_s3"},
    {128, 128, "igemm_fwd_ws_128x128x64_4w2f_s4", "igemm_dgrad_ws_128x128x64_4w2f_s4"},
    {256, 256, "igemm_fwd_ws_256x256x64_8w0f_s2", "igemm_dgrad_ws_256x256x64_8w0f_s2"},
    {256, 128, "igemm_fwd_ws_256x128x64_8w2f_s3", "igemm_dgrad_ws_256x128x64_8w2f_s3"},
    {128, 128, "igemm_fwd_ws_128x128x64_8w2f_s3", "igemm_dgrad_ws_128x128x64_8w2f_s3"},
    {128, 128, "igemm_fwd_ws_128x128x64_8w0f_s3", "igemm_dgrad_ws_128x128x64_8w0f_s3"},
    {256, 128, "igemm_fwd_ws_256x128x64_8w0f_s3", "igemm_dgrad_ws_256x128x64_8w0f_s3"},
    {128, 64, "igemm_fwd_ws_128x64x64_4w2f_s4", "igemm_dgrad_ws_128x64x64_4w2f_s4"},
    {128, 64, "igemm_fwd_ws_128x64x64_8w0f_s4", "igemm_dgrad_ws_128x64x64_8w0f_s4"},
    {128, 256, "igemm_fwd_ws_128x256x64_8w0f_s3", "igemm_dgrad_ws_128x256x64_8w0f_s3"},
    {224, 256, "igemm_fwd_ws_224x256x64_8w0f_s2_m16", "igemm_dgrad_ws_224x256x64_8w0f_s2_m16"},
    {256, 256, "igemm_fwd_ws_256x256x64_8w0f_s2_m16", "igemm_dgrad_ws_256x256x64_8w0f_s2_m16"},
    {128, 128, "igemm_fwd_ws_128x128x64_4w2f_s3_m16", "igemm_dgrad_ws_128x128x64_4w2f_s3_m16"},
    {256, 128, "igemm_fwd_ws_256x128x64_8w2f_s3_m16", "igemm_dgrad_ws_256x128x64_8w2f_s3_m16"},
    {256, 128, "igemm_fwd_ws_256x128x64_8w0f_s3_m16", "igemm_dgrad_ws_256x128x64_8w0f_s3_m16"},
    {128, 256, "igemm_fwd_ws_128x256x64_8w0f_s3_m16", "igemm_dgrad_ws_128x256x64_8w0f_s3_m16"},
    {224, 128, "igemm_fwd_ws_224x128x64_8w0f_s3_m16", "igemm_dgrad_ws_224x128x64_8w0f_s3_m16"},
    {64, 64, "igemm_fwd_ws_64x64x64_4w2f_s4", "igemm_dgrad_ws_64x64x64_4w2f_s4"},
    {64, 128, "igemm_fwd_ws_64x128x64_4w2f_s4", "igemm_dgrad_ws_64x128x64_4w2f_s4"},
    {64, 64, "igemm_fwd_ws_64x64x64_4w2f_s4_m16", "igemm_dgrad_ws_64x64x64_4w2f_s4_m16"},
    {64, 128, "igemm_fwd_ws_64x128x64_4w2f_s4_m16", "igemm_dgrad_ws_64x128x64_4w2f_s4_m16"},
    {144, 128, "igemm_fwd_ws_144x128x64_6w2f_s3_m16", "igemm_dgrad_ws_144x128x64_6w2f_s3_m16"},
    {144, 256, "igemm_fwd_ws_144x256x64_6w2f_s2_m16", "igemm_dgrad_ws_144x256x64_6w2f_s2_m16"},
    {144, 64, "igemm_fwd_ws_144x64x64_3w2f_s4_m16", "igemm_dgrad_ws_144x64x64_3w2f_s4_m16"},
    {224, 256, "igemm_fwd_ws_224x256x64_8w0f_s2_m16_tail128", "igemm_dgrad_ws_224x256x64_8w0f_s2_m16_tail128"},
};

#define SDCONV_WS_CASE(idx, BM, BN, WGM, WGN, S, BK, NP)                                      \
    case 2 * (idx): return launch_ws_variant<0, BM, BN, WGM, WGN, S, BK, NP>(P, st);          \
    case 2 * (idx) + 1: return launch_ws_variant<1, BM, BN, WGM, WGN, S, BK, NP>(P, st);

hipError_t launch_igemm_ws(int variant, const IgemmParams& P, hipStream_t st)
{
    const int key = variant * 2 + (P.mode ? 1 : 0);
    switch (key) {
        SDCONV_WS_CASE(0, 128, 128, 2, 2, 3, 64, 2)
        SDCONV_WS_CASE(1, 128, 128, 2, 2, 4, 64, 2)
        SDCONV_WS_CASE(2, 256, 256, 2, 4, 2, 64, 0)
        SDCONV_WS_CASE(3, 256, 128, 4, 2, 3, 64, 2)
        SDCONV_WS_CASE(4, 128, 128, 2, 4, 3, 64, 2)
        SDCONV_WS_CASE(5, 128, 128, 2, 4, 3, 64, 0)
        SDCONV_WS_CASE(6, 256, 128, 4, 2, 3, 64, 0)
        SDCONV_WS_CASE(7, 128, 64, 2, 2, 4, 64, 2)
        SDCONV_WS_CASE(8, 128, 64, 4, 2, 4, 64, 0)
        SDCONV_WS_CASE(9, 128, 256, 2, 4, 3, 64, 0)
        case 20: return launch_ws_variant<0, 224, 256, 2, 4, 2, 64, 0, 16>(P, st);
        case 21: return launch_ws_variant<1, 224, 256, 2, 4, 2, 64, 0, 16>(P, st);
        case 22: return launch_ws_variant<0, 256, 256, 2, 4, 2, 64, 0, 16>(P, st);
        case 23: return launch_ws_variant<1, 256, 256, 2, 4, 2, 64, 0, 16>(P, st);
        case 24: return launch_ws_variant<0, 128, 128, 2, 2, 3, 64, 2, 16>(P, st);
        case 25: return launch_ws_variant<1, 128, 128, 2, 2, 3, 64, 2, 16>(P, st);
        case 26: return launch_ws_variant<0, 256, 128, 4, 2, 3, 64, 2, 16>(P, st);
        case 27: return launch_ws_variant<1, 256, 128, 4, 2, 3, 64, 2, 16>(P, st);
        case 28: return launch_ws_variant<0, 256, 128, 4, 2, 3, 64, 0, 16>(P, st);
        case 29: return launch_ws_variant<1, 256, 128, 4, 2, 3, 64, 0, 16>(P, st);
        case 30: return launch_ws_variant<0, 128, 256, 2, 4, 3, 64, 0, 16>(P, st);
        case 31: return launch_ws_variant<1, 128, 256, 2, 4, 3, 64, 0, 16>(P, st);
        case 32: return launch_ws_variant<0, 224, 128, 2, 4, 3, 64, 0, 16>(P, st);
        case 33: return launch_ws_variant<1, 224, 128, 2, 4, 3, 64, 0, 16>(P, st);
        // small tiles: layers with few pixels (res5 on a 25x42 map, fully connected heads) still
        // give every compute unit a workgroup
        case 34: return launch_ws_variant<0, 64, 64, 2, 2, 4, 64, 2>(P, st);
        case 35: return launch_ws_variant<1, 64, 64, 2, 2, 4, 64, 2>(P, st);
        case 36: return launch_ws_variant<0, 64, 128, 2, 2, 4, 64, 2>(P, st);
        case 37: return launch_ws_variant<1, 64, 128, 2, 2, 4, 64, 2>(P, st);
        case 38: return launch_ws_variant<0, 64, 64, 2, 2, 4, 64, 2, 16>(P, st);
        case 39: return launch_ws_variant<1, 64, 64, 2, 2, 4, 64, 2, 16>(P, st);
        case 40: return launch_ws_variant<0, 64, 128, 2, 2, 4, 64, 2, 16>(P, st);
        case 41: return launch_ws_variant<1, 64, 128, 2, 2, 4, 64, 2, 16>(P, st);
        // 144-row tiles (three wave rows of 48): the 8400 / 33600 / 134400 pixel rows of the backbone
        // stages make 59 / 234 / 934 of them, which fill 256 compute units to 91-92 % where 128-row
        // tiles fill 52-69 %
        case 42: return launch_ws_variant<0, 144, 128, 3, 2, 3, 64, 2, 16>(P, st);
        case 43: return launch_ws_variant<1, 144, 128, 3, 2, 3, 64, 2, 16>(P, st);
        case 44: return launch_ws_variant<0, 144, 256, 3, 2, 2, 64, 2, 16>(P, st);
        case 45: return launch_ws_variant<1, 144, 256, 3, 2, 2, 64, 2, 16>(P, st);
        case 46: return launch_ws_variant<0, 144, 64, 3, 1, 4, 64, 2, 16>(P, st);
        case 47: return launch_ws_variant<1, 144, 64, 3, 1, 4, 64, 2, 16>(P, st);
        // 224 x 256 tiles for the whole rounds of 256 workgroups, 224 x 128 for the rest
        case 48: return launch_ws_mixed<0, 224, 256, 128, 2, 4, 2, 3, 64, 16>(P, st);
        case 49: return launch_ws_mixed<1, 224, 256, 128, 2, 4, 2, 3, 64, 16>(P, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sdconv
