// Parameters of the implicit-GEMM forward / data-gradient kernel.
#pragma once
#include "common.h"

namespace sdconv {

constexpr int kMaxTaps = 64;      // R*S the MFMA route accepts
constexpr int kMaxClasses = 16;   // stride_h*stride_w parity classes of a strided dgrad

struct IgemmParams {
    const __half* A;   // gathered activations: x (forward) or dy (data gradient)
    const __half* B;   // filter matrix, one row per destination channel: [Cd][R][S][Cs]
    __half* D;         // destination activations
    int NB;            // batch
    int Hs, Ws, Cs;    // source image extents and channels (contraction channels per tap)
    int Hd, Wd, Cd;    // destination image extents and channels
    int R, S;
    int sh, sw, ph, pw, dh, dw;
    int mode;          // 0 forward, 1 data gradient
    int nclasses;      // 1, or stride_h*stride_w for a data gradient
    int sw_cls;        // classes along w (stride_w for a data gradient, else 1)
    int tiles_n;       // column tiles
    int total_tiles;   // row tiles (all classes) x column tiles
    int b_row_pitch;   // R*S*Cs
    int class_tile_start[kMaxClasses + 1];   // first row-tile of each class, then the total
    int tiles_h, tiles_w;   // spatial tiles per image (patch kernels only)
    // launches with two tile widths (igemm_ws_mixed_kernel; set by its launcher)
    int mix_big_tiles, mix_big_blocks;                        // wide tiles, and the workgroups that cover them
    int mix_small_tiles, mix_small_tiles_n, mix_small_tm0;    // narrow tiles: count, per row tile, first row tile
    Epilogue ep;            // elementwise tail before the rounding to binary16 (all null: none)
};

struct IgemmVariant { int bm, bn; const char* fwd_name; const char* dgrad_name; };
constexpr int kNumIgemmVariants = 4;
extern const IgemmVariant kIgemmVariants[kNumIgemmVariants];

constexpr int kNumIgemmDmaVariants = 14;
extern const IgemmVariant kIgemmDmaVariants[kNumIgemmDmaVariants];
hipError_t launch_igemm_dma(int variant, const IgemmParams& P, hipStream_t st);
constexpr int kNumIgemmWsVariants = 25;
extern const IgemmVariant kIgemmWsVariants[kNumIgemmWsVariants];
hipError_t launch_igemm_ws(int variant, const IgemmParams& P, hipStream_t st);
struct PatchVariant { int th, tw, bn, tps, stages; const char* fwd_name; const char* dgrad_name; int one_slab = 0; };
// tps: taps per pipeline step, must divide R*S, and R*S/tps must be at least stages-1;
// one_slab: the variant has a single patch buffer and takes layers with 64 source channels only
constexpr int kNumPatchVariants = 36;
extern const PatchVariant kPatchVariants[kNumPatchVariants];
hipError_t launch_conv_patch(int variant, const IgemmParams& P, hipStream_t st);
hipError_t launch_igemm(int variant, const IgemmParams& P, int total_tiles, hipStream_t st);
hipError_t launch_filter_transpose(const __half* w, __half* wT, int K, int RS, int C, hipStream_t st);

}  // namespace sdconv
