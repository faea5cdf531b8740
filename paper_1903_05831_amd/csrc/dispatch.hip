// Kernel selection: which route and tile variant serves a given geometry and pass.
#include "common.h"
#include "igemm.h"
#include "wgrad.h"
#include "thin.h"
#include <stdlib.h>
#include <map>
#include <mutex>
#include <string>

namespace sdconv {

static int env_int(const char* name, int dflt)
{
    const char* e = getenv(name);
    return (e && *e) ? atoi(e) : dflt;
}

// Tuning hooks (used by the tuner and by the tests that force every variant): environment
// variables that override the dispatcher, honoured only when SDCONV_TUNE=1 was set before the
// library's first call.  That switch is read once; without it no call touches the environment.
static bool tuning()
{
    static const bool on = env_int("SDCONV_TUNE", 0) != 0;
    return on;
}
static int hook(const char* name, int dflt) { return tuning() ? env_int(name, dflt) : dflt; }

static bool force_direct() { return hook("SDCONV_FORCE_DIRECT", 0) != 0; }
static int forced_variant() { return hook("SDCONV_IGEMM_VARIANT", -1); }
static int forced_wgrad_splits() { return hook("SDCONV_WGRAD_SPLITS", -1); }
static int forced_wgrad_variant() { return hook("SDCONV_WGRAD_VARIANT", -1); }

static size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

// Measured choices for known geometries (written by tune.py on the target GPU); anything not
// listed falls back to the heuristics below.
struct TunedEntry { int N, H, W, C, K, R, S, sh, sw, ph, pw, dh, dw, pass, variant, splits; };
static const TunedEntry kTuned[] = {
#include "tuned_table.inc"
    {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, -1, 0, 0},
};

// The table was measured at the batch sizes of the detector workloads.  A layer with the same
// geometry and a batch within a factor of two of a measured one (half or twice the rows: the same
// tile shapes still fill the chip about as well) takes that entry too, the exact batch first;
// *scale_splits is then the factor by which the pixel count, and with it the number of pixel
// ranges of a weight gradient, differs from the measured one.
static const TunedEntry* tuned_lookup(const Geom& g, int pass, double* scale_splits = nullptr)
{
    if (hook("SDCONV_NO_TUNED_TABLE", 0)) return nullptr;
    const TunedEntry* near = nullptr;
    for (const TunedEntry* e = kTuned; e->pass >= 0; ++e) {
        if (!(e->pass == pass && e->H == g.H && e->W == g.W && e->C == g.C && e->K == g.K &&
              e->R == g.R && e->S == g.S && e->sh == g.sh && e->sw == g.sw && e->ph == g.ph && e->pw == g.pw &&
              e->dh == g.dh && e->dw == g.dw))
            continue;
        if (e->N == g.N) { near = e; break; }
        if (!near && 2 * g.N >= e->N && g.N <= 2 * e->N) near = e;
    }
    if (near && scale_splits) *scale_splits = (double)g.N / near->N;
    return near;
}

// The LDS-DMA kernels address their binary16 operands with 32-bit BYTE offsets and use bit 31
// of the offset as "outside the image / past the tile" (the hardware range check then writes
// zeros).  A tensor of 2^30 elements or more has real data at such offsets, so a masked load
// would fetch it instead of zeros: those layers take the register-staged kernels (igemm.hip,
// wgrad.hip), which index elements and test every load themselves.
static bool byte_offsets_fit_31_bits(const Geom& g)
{
    const long lim = 1L << 30;
    return (long)g.N * g.H * g.W * g.C < lim && (long)g.N * g.Ho * g.Wo * g.K < lim &&
           (long)g.K * g.R * g.S * g.C < lim;
}

// The MFMA route moves 16-byte (8-half) vectors along the channel axis of every tensor.
static bool igemm_ok(const Geom& g)
{
    if (force_direct()) return false;
    if (g.C % 8 || g.K % 8) return false;
    if (g.R * g.S > kMaxTaps) return false;
    return true;
}

// Row tiles of the fwd/dgrad index space for a tile height bm.
static int row_tiles(const Geom& g, bool dgrad, int bm, int* starts, int* nclasses)
{
    if (!dgrad) {
        long M = (long)g.N * g.Ho * g.Wo;
        starts[0] = 0;
        starts[1] = (int)((M + bm - 1) / bm);
        *nclasses = 1;
        return starts[1];
    }
    int nc = g.sh * g.sw, acc = 0;
    for (int q = 0; q < nc; ++q) {
        int a = q / g.sw, b = q % g.sw;
        long Hi = (g.H - a + g.sh - 1) / g.sh, Wj = (g.W - b + g.sw - 1) / g.sw;
        if (Hi < 0) Hi = 0;
        if (Wj < 0) Wj = 0;
        long M = (long)g.N * Hi * Wj;
        starts[q] = acc;
        acc += (int)((M + bm - 1) / bm);
    }
    starts[nc] = acc;
    *nclasses = nc;
    return acc;
}

static const IgemmVariant& igemm_variant(int v)
{
    if (v >= 300) return kIgemmWsVariants[v - 300];
    return v >= 100 ? kIgemmDmaVariants[v - 100] : kIgemmVariants[v];
}

// The patch kernels take stride-1 layers whose taps span exactly two extra rows and columns
// (3x3, dilation 1) and whose contraction channels come in whole 64-channel slabs.
static bool patch_ok(const Geom& g, bool dgrad)
{
    int cs = dgrad ? g.K : g.C;
    return g.sh == 1 && g.sw == 1 && (g.R - 1) * g.dh == 2 && (g.S - 1) * g.dw == 2 && cs % 64 == 0 &&
           g.R * g.S >= 4;
}

static bool patch_variant_ok(const Geom& g, bool dgrad, int v)
{
    const PatchVariant& pv = kPatchVariants[v - 400];
    const int taps = g.R * g.S;
    if (pv.one_slab && (dgrad ? g.K : g.C) != 64) return false;
    return patch_ok(g, dgrad) && taps % pv.tps == 0 && taps / pv.tps >= pv.stages - 1;
}

static const char* igemm_name(int v, bool dgrad)
{
    if (v >= 400) return dgrad ? kPatchVariants[v - 400].dgrad_name : kPatchVariants[v - 400].fwd_name;
    return dgrad ? igemm_variant(v).dgrad_name : igemm_variant(v).fwd_name;
}

// The launch with two tile widths (324) takes undivided images only: a strided data gradient
// with its parity classes runs as the plain 224 x 256 variant.
static int ws_variant_for(const Geom& g, bool dgrad, int v)
{
    if (v == 324 && dgrad && g.sh * g.sw > 1) return 310;
    return v;
}

static int pick_variant(const Geom& g, bool dgrad)
{
    if (!byte_offsets_fit_31_bits(g)) return (dgrad ? g.C : g.K) <= 64 ? 3 : 0;
    int fv = forced_variant();
    if (fv >= 400 && fv < 400 + kNumPatchVariants && patch_variant_ok(g, dgrad, fv)) return fv;
    if (fv >= 400) fv = -1;
    if (fv >= 0 && fv < kNumIgemmVariants) return fv;
    if (fv >= 100 && fv < 100 + kNumIgemmDmaVariants) return fv;
    if (fv >= 300 && fv < 300 + kNumIgemmWsVariants) return ws_variant_for(g, dgrad, fv);
    if (const TunedEntry* e = tuned_lookup(g, dgrad ? SDCONV_DGRAD : SDCONV_FWD))
        if (e->variant < 400 || patch_variant_ok(g, dgrad, e->variant)) return ws_variant_for(g, dgrad, e->variant);
    // No table entry: rules read off the tuned layers of the detector workloads.
    const int nout = dgrad ? g.C : g.K;
    const int kgemm = g.R * g.S * (dgrad ? g.K : g.C);
    const long rows = dgrad ? (long)g.N * g.H * g.W : (long)g.N * g.Ho * g.Wo;
    int starts[kMaxClasses + 1], nc;
    // stride-1 3x3-class layers: the patch-resident kernel (wide blocks when there is enough work),
    // unless its 10x14 pixel blocks would be mostly empty (the 7x7 maps of an RoI head)
    const int Hd = dgrad ? g.H : g.Ho, Wd = dgrad ? g.W : g.Wo;
    const long covered = (long)((Hd + 9) / 10) * 10 * ((Wd + 13) / 14) * 14;
    const bool blocks_fill = covered * 2 <= (long)Hd * Wd * 3;      // at most 1.5x the pixels
    if (blocks_fill && nout >= 128 && rows >= 20000 && patch_variant_ok(g, dgrad, 415)) return 415;
    if (blocks_fill && (dgrad ? g.K : g.C) == 64 && patch_variant_ok(g, dgrad, 433)) return 433;
    if (blocks_fill && patch_variant_ok(g, dgrad, 429)) return 429;
    // narrow outputs: 64-wide tiles
    if (nout <= 64) return 100 + 7;
    // enough rows to fill the chip with 224-row tiles: the big tile for long contractions and wide
    // outputs (half the LDS traffic per flop), else the 128-wide one; small layers: 128x128
    const int t224 = row_tiles(g, dgrad, 224, starts, &nc);
    if (kgemm >= 512 && nout >= 256 && (long)t224 * ((nout + 255) / 256) >= 200) return 300 + 10;
    if ((long)t224 * ((nout + 127) / 128) >= 200) return 300 + 16;
    // few pixels (a 25x42 map, a fully connected head): small tiles, so that every compute unit
    // still gets a workgroup
    const long t128 = (long)row_tiles(g, dgrad, 128, starts, &nc) * ((nout + 127) / 128);
    if (t128 < 160) {
        const long t64x128 = (long)row_tiles(g, dgrad, 64, starts, &nc) * ((nout + 127) / 128);
        return t64x128 >= 200 ? 300 + 20 : 300 + 19;
    }
    return 300 + 0;
}

static bool thin_ok(const Geom& g) { return !force_direct() && g.C <= 4 && thin_supported(g); }

// Filter counts that are not a multiple of 8 (with channels that are): the layer runs as one with
// the filter count rounded up, on padded copies of the filter and of the K-channel tensor that
// live in the workspace (padk.hip).
static bool padk_ok(const Geom& g)
{
    if (force_direct() || hook("SDCONV_NO_PADK", 0)) return false;
    if (g.K % 8 == 0 || g.C % 8 != 0 || g.R * g.S > kMaxTaps || g.sh * g.sw > kMaxClasses) return false;
    // the padded copies must stay below 2^31 elements like every other tensor
    const long kp = (g.K + 7) / 8 * 8, lim = 0x7fffffffL;
    return (long)g.N * g.Ho * g.Wo * kp <= lim && kp * g.R * g.S * g.C <= lim;
}
static Geom padded_k(const Geom& g) { Geom p = g; p.K = (g.K + 7) / 8 * 8; return p; }
static size_t padk_filter_bytes(const Geom& gp) { return align256((size_t)gp.K * gp.R * gp.S * gp.C * sizeof(__half)); }
static size_t padk_act_bytes(const Geom& gp) { return align256((size_t)gp.N * gp.Ho * gp.Wo * gp.K * sizeof(__half)); }
static size_t padk_dw_bytes(const Geom& gp) { return align256((size_t)gp.K * gp.R * gp.S * gp.C * sizeof(float)); }

// "padk+<inner kernel name>", kept for the life of the process
static const char* padk_name(const char* inner)
{
    static std::mutex mu;
    static std::map<std::string, std::string> names;
    std::lock_guard<std::mutex> lock(mu);
    auto it = names.find(inner);
    if (it == names.end()) it = names.emplace(inner, std::string("padk+") + inner).first;
    return it->second.c_str();
}

Plan plan_fwd(const Geom& g)
{
    if (padk_ok(g)) {
        const Geom gp = padded_k(g);
        const Plan in = plan_fwd(gp);
        return Plan{ROUTE_PADK, in.variant, 1, padk_filter_bytes(gp) + padk_act_bytes(gp) + in.workspace_bytes,
                    padk_name(in.name)};
    }
    if (thin_ok(g)) return Plan{ROUTE_THIN, 0, 1, align256(thin_packed_filter_bytes(g)), "thin_fwd"};
    if (!igemm_ok(g)) return Plan{ROUTE_DIRECT, 0, 1, 0, "direct_fwd"};
    int v = pick_variant(g, false);
    return Plan{ROUTE_IGEMM, v, 1, 0, igemm_name(v, false)};
}

Plan plan_dgrad(const Geom& g)
{
    if (padk_ok(g)) {
        const Geom gp = padded_k(g);
        const Plan in = plan_dgrad(gp);
        return Plan{ROUTE_PADK, in.variant, 1, padk_filter_bytes(gp) + padk_act_bytes(gp) + in.workspace_bytes,
                    padk_name(in.name)};
    }
    if (!force_direct() && g.C <= 4 && thin_dgrad_mfma_supported(g) && byte_offsets_fit_31_bits(g) &&
        !hook("SDCONV_NO_THIN_MFMA_DGRAD", 0))
        return Plan{ROUTE_THIN, 1, 1, align256(thin_dgrad_mfma_workspace_bytes(g)), "thin_dgrad_mfma"};
    if (!force_direct() && g.C <= 4 && g.K % 8 == 0 && g.sh * g.sw <= kMaxClasses &&
        thin_dgrad_lds_bytes(g) <= 64 * 1024)
        return Plan{ROUTE_THIN, 0, 1, align256((size_t)g.K * g.R * g.S * g.C * sizeof(__half)), "thin_dgrad"};
    if (!igemm_ok(g) || g.sh * g.sw > kMaxClasses) return Plan{ROUTE_DIRECT, 0, 1, 0, "direct_dgrad"};
    int v = pick_variant(g, true);
    // the older kernels want the filter transposed to [C][R][S][K] in the workspace; the
    // split-role and patch kernels read it as stored
    size_t ws = v >= 300 ? 0 : align256((size_t)g.K * g.R * g.S * g.C * sizeof(__half));
    return Plan{ROUTE_IGEMM, v, 1, ws, igemm_name(v, true)};
}

// Pixel-range count for the weight gradient: enough workgroups to fill the chip a few times
// over, but at least four 64-pixel steps per range.
static const WgradVariant& wgrad_variant(int v)
{
    return v >= 100 ? kWgradDmaVariants[v - 100] : kWgradVariants[v];
}

static int pick_wgrad_variant(const Geom& g)
{
    if (!byte_offsets_fit_31_bits(g)) return g.K <= 64 ? 1 : 0;
    int fv = forced_wgrad_variant();
    if ((fv >= 0 && fv < kNumWgradVariants) || (fv >= 100 && fv < 100 + kNumWgradDmaVariants)) return fv;
    if (const TunedEntry* e = tuned_lookup(g, SDCONV_WGRAD)) return e->variant;
    // No table entry: rules read off the tuned layers of the detector workloads (tile = filters x
    // channels of one tap): narrow tiles for narrow layers, the 256x256 tile when both are wide
    // and the pixel axis is long enough to feed it, else 128x128.
    const long pixels = (long)g.N * g.Ho * g.Wo;
    if (g.K <= 64 && g.C <= 64) return 100 + 7;
    if (g.K <= 64) return 100 + 20;
    if (g.C <= 64) return 100 + 8;
    if (g.K >= 512 && g.C >= 512 && pixels >= 20000) return 100 + 14;
    return 100 + 12;
}

static void wgrad_split(const Geom& g, int variant, int* splits, int* steps_per_split)
{
    const WgradVariant& v = wgrad_variant(variant);
    long tiles = (long)((g.K + v.bm - 1) / v.bm) * ((g.C + v.bn - 1) / v.bn) * g.R * g.S;
    long P = (long)g.N * g.Ho * g.Wo;
    long total_steps = (P + 63) / 64;
    long want = (384 + tiles - 1) / tiles;
    double scale = 1.0;
    if (const TunedEntry* e = tuned_lookup(g, SDCONV_WGRAD, &scale)) want = (long)(e->splits * scale + 0.5);
    int fs = forced_wgrad_splits();
    if (fs > 0) want = fs;
    long cap = total_steps / 4;
    if (cap < 1) cap = 1;
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    long sps = (total_steps + want - 1) / want;
    *steps_per_split = (int)sps;
    *splits = (int)((total_steps + sps - 1) / sps);
}

Plan plan_wgrad(const Geom& g)
{
    if (padk_ok(g)) {
        const Geom gp = padded_k(g);
        const Plan in = plan_wgrad(gp);
        return Plan{ROUTE_PADK, in.variant, in.splits, padk_act_bytes(gp) + padk_dw_bytes(gp) + in.workspace_bytes,
                    padk_name(in.name)};
    }
    if (thin_ok(g)) return Plan{ROUTE_THIN, 0, 1, align256(thin_wgrad_partial_bytes(g)), "thin_wgrad"};
    if (!igemm_ok(g)) return Plan{ROUTE_DIRECT, 0, 1, 0, "direct_wgrad"};
    int v = pick_wgrad_variant(g);
    int splits, sps;
    wgrad_split(g, v, &splits, &sps);
    size_t ws = splits > 1 ? align256((size_t)splits * g.K * g.R * g.S * g.C * sizeof(float)) : 0;
    Plan p{ROUTE_IGEMM, v, splits, ws, wgrad_variant(v).name};
    p.steps_per_split = sps;
    return p;
}

static hipError_t run_igemm(const Geom& g, const Plan& p, bool dgrad, const __half* A, const __half* B,
                            __half* D, hipStream_t st, const Epilogue& ep)
{
    IgemmParams P;
    P.ep = ep;
    P.A = A; P.B = B; P.D = D;
    P.NB = g.N;
    if (!dgrad) { P.Hs = g.H; P.Ws = g.W; P.Cs = g.C; P.Hd = g.Ho; P.Wd = g.Wo; P.Cd = g.K; }
    else        { P.Hs = g.Ho; P.Ws = g.Wo; P.Cs = g.K; P.Hd = g.H; P.Wd = g.W; P.Cd = g.C; }
    P.R = g.R; P.S = g.S;
    P.sh = g.sh; P.sw = g.sw; P.ph = g.ph; P.pw = g.pw; P.dh = g.dh; P.dw = g.dw;
    P.mode = dgrad ? 1 : 0;
    P.sw_cls = dgrad ? g.sw : 1;
    // elements between consecutive rows of the filter matrix the kernel reads: [Cd][R][S][Cs]
    // (forward, and the transposed copy of the older data-gradient kernels), or the filter as
    // stored, [K = Cs][R][S][C = Cd], for the data gradient of the split-role and patch kernels
    P.b_row_pitch = g.R * g.S * ((dgrad && p.variant >= 300) ? P.Cd : P.Cs);
    P.tiles_h = P.tiles_w = 0;
    if (p.variant >= 400) {
        const PatchVariant& pv = kPatchVariants[p.variant - 400];
        P.nclasses = 1;
        P.class_tile_start[0] = 0;
        P.tiles_h = (P.Hd + pv.th - 1) / pv.th;
        P.tiles_w = (P.Wd + pv.tw - 1) / pv.tw;
        P.tiles_n = (P.Cd + pv.bn - 1) / pv.bn;
        P.total_tiles = P.NB * P.tiles_h * P.tiles_w * P.tiles_n;
        P.class_tile_start[1] = P.total_tiles;
        return launch_conv_patch(p.variant - 400, P, st);
    }
    const IgemmVariant& v = igemm_variant(p.variant);
    int tiles_m = row_tiles(g, dgrad, v.bm, P.class_tile_start, &P.nclasses);
    P.tiles_n = (P.Cd + v.bn - 1) / v.bn;
    P.total_tiles = tiles_m * P.tiles_n;
    if (p.variant >= 300) return launch_igemm_ws(p.variant - 300, P, st);
    if (p.variant >= 100) return launch_igemm_dma(p.variant - 100, P, st);
    return launch_igemm(p.variant, P, P.total_tiles, st);
}

hipError_t run_fwd(const Geom& g, const Plan& p, const __half* x, const __half* w, __half* y, void* ws, hipStream_t st,
                   const Epilogue& ep)
{
    if (p.route == ROUTE_PADK) {
        // zero filters behind the real ones; the padded result goes to the workspace and its real
        // channels are copied out (with the tail, if any: it sees the rounded result there)
        const Geom gp = padded_k(g);
        unsigned char* base = static_cast<unsigned char*>(ws);
        __half* wp = reinterpret_cast<__half*>(base);
        __half* yp = reinterpret_cast<__half*>(base + padk_filter_bytes(gp));
        void* inner_ws = base + padk_filter_bytes(gp) + padk_act_bytes(gp);
        const long wn = (long)g.K * g.R * g.S * g.C, wpn = (long)gp.K * g.R * g.S * g.C;
        hipError_t e = launch_pad_rows(w, wp, wn, wpn, st);
        if (e != hipSuccess) return e;
        e = run_fwd(gp, plan_fwd(gp), x, wp, yp, inner_ws, st, no_epilogue());
        if (e != hipSuccess) return e;
        return launch_unpad_channels(yp, y, (long)g.N * g.Ho * g.Wo, g.K, gp.K, ep, st);
    }
    if (p.route == ROUTE_DIRECT) return launch_direct_fwd(g, x, w, y, st, ep);
    if (p.route == ROUTE_THIN) return launch_thin_fwd(g, x, w, y, ws, st, ep);
    return run_igemm(g, p, false, x, w, y, st, ep);
}

hipError_t run_dgrad(const Geom& g, const Plan& p, const __half* dy, const __half* w, __half* dx, void* ws, hipStream_t st,
                     const Epilogue& ep)
{
    if (p.route == ROUTE_PADK) {
        // zero gradient channels and zero filters behind the real ones; dx comes out in place
        const Geom gp = padded_k(g);
        unsigned char* base = static_cast<unsigned char*>(ws);
        __half* wp = reinterpret_cast<__half*>(base);
        __half* gpad = reinterpret_cast<__half*>(base + padk_filter_bytes(gp));
        void* inner_ws = base + padk_filter_bytes(gp) + padk_act_bytes(gp);
        const long wn = (long)g.K * g.R * g.S * g.C, wpn = (long)gp.K * g.R * g.S * g.C;
        hipError_t e = launch_pad_rows(w, wp, wn, wpn, st);
        if (e != hipSuccess) return e;
        e = launch_pad_channels(dy, gpad, (long)g.N * g.Ho * g.Wo, g.K, gp.K, st);
        if (e != hipSuccess) return e;
        return run_dgrad(gp, plan_dgrad(gp), gpad, wp, dx, inner_ws, st, ep);
    }
    if (p.route == ROUTE_DIRECT) return launch_direct_dgrad(g, dy, w, dx, st, ep);
    if (p.route == ROUTE_THIN && p.variant == 1) return launch_thin_dgrad_mfma(g, dy, w, dx, ws, st, ep);
    if (p.route == ROUTE_IGEMM && p.variant >= 300) return run_igemm(g, p, true, dy, w, dx, st, ep);
    __half* wT = static_cast<__half*>(ws);
    hipError_t e = launch_filter_transpose(w, wT, g.K, g.R * g.S, g.C, st);
    if (e != hipSuccess) return e;
    if (p.route == ROUTE_THIN) return launch_thin_dgrad(g, dy, wT, dx, st, ep);
    return run_igemm(g, p, true, dy, wT, dx, st, ep);
}

hipError_t run_wgrad(const Geom& g, const Plan& p, const __half* x, const __half* dy, float* dw, void* ws, hipStream_t st)
{
    if (p.route == ROUTE_PADK) {
        // zero gradient channels behind the real ones; the first K filters of the padded result are dw
        const Geom gp = padded_k(g);
        unsigned char* base = static_cast<unsigned char*>(ws);
        __half* gpad = reinterpret_cast<__half*>(base);
        float* dwp = reinterpret_cast<float*>(base + padk_act_bytes(gp));
        void* inner_ws = base + padk_act_bytes(gp) + padk_dw_bytes(gp);
        hipError_t e = launch_pad_channels(dy, gpad, (long)g.N * g.Ho * g.Wo, g.K, gp.K, st);
        if (e != hipSuccess) return e;
        e = run_wgrad(gp, plan_wgrad(gp), x, gpad, dwp, inner_ws, st);
        if (e != hipSuccess) return e;
        return launch_copy_f32(dwp, dw, (long)g.K * g.R * g.S * g.C, st);
    }
    if (p.route == ROUTE_DIRECT) return launch_direct_wgrad(g, x, dy, dw, st);
    if (p.route == ROUTE_THIN) return launch_thin_wgrad(g, x, dy, dw, ws, st);
    const WgradVariant& v = wgrad_variant(p.variant);
    WgradParams P;
    P.X = x; P.G = dy;
    P.N = g.N; P.H = g.H; P.W = g.W; P.C = g.C; P.K = g.K; P.R = g.R; P.S = g.S;
    P.sh = g.sh; P.sw = g.sw; P.ph = g.ph; P.pw = g.pw; P.dh = g.dh; P.dw = g.dw;
    P.Ho = g.Ho; P.Wo = g.Wo;
    P.P = g.N * g.Ho * g.Wo;
    P.splits = p.splits;
    P.steps_per_split = p.steps_per_split;
    P.tiles_k = (g.K + v.bm - 1) / v.bm;
    P.tiles_c = (g.C + v.bn - 1) / v.bn;
    P.out = (P.splits > 1) ? static_cast<float*>(ws) : dw;
    hipError_t e = p.variant >= 100 ? launch_wgrad_dma(p.variant - 100, P, st) : launch_wgrad(p.variant, P, st);
    if (e != hipSuccess || P.splits == 1) return e;
    return launch_splitk_reduce(static_cast<const float*>(ws), dw, P.splits, (long)g.K * g.R * g.S * g.C, st);
}

}  // namespace sdconv
