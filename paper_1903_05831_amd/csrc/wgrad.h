// Parameters of the split-K weight-gradient kernels.
#pragma once
#include "common.h"

namespace sdconv {

struct WgradParams {
    const __half* X;    // activations [N][H][W][C]
    const __half* G;    // upstream gradient [N][Ho][Wo][K]
    float* out;         // dw when splits == 1, else the partial-sum workspace [splits][K][R][S][C]
    int N, H, W, C, K, R, S;
    int sh, sw, ph, pw, dh, dw;
    int Ho, Wo;
    int P;              // N*Ho*Wo, the contraction length
    int splits;         // pixel ranges
    int steps_per_split;  // 64-pixel steps each split covers
    int tiles_k, tiles_c; // filter tiles, channel tiles (per tap)
    int total_blocks;     // tiles_c * tiles_k * R * S * splits (set by the launcher)
};

struct WgradVariant { int bm, bn; const char* name; };
constexpr int kNumWgradVariants = 2;
extern const WgradVariant kWgradVariants[kNumWgradVariants];

constexpr int kNumWgradDmaVariants = 21;
extern const WgradVariant kWgradDmaVariants[kNumWgradDmaVariants];
hipError_t launch_wgrad_dma(int variant, const WgradParams& P, hipStream_t st);
hipError_t launch_wgrad(int variant, const WgradParams& P, hipStream_t st);
hipError_t launch_splitk_reduce(const float* partial, float* dw, int splits, long numel, hipStream_t st);

}  // namespace sdconv
