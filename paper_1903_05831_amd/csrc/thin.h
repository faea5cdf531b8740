// Parameters of the thin-input (C <= 4) stem kernels.
#pragma once
#include "common.h"

namespace sdconv {

struct ThinParams {
    const __half* X;     // input [N][H][W][C], C <= 4
    const __half* Wp;    // packed filter bank (forward)
    __half* Y;           // forward output
    const __half* G;     // upstream gradient (wgrad)
    float* partial;      // wgrad partial sums
    int N, H, W, C, K, R, S;
    int sh, sw, ph, pw, Ho, Wo;
    int tiles_h, tiles_w, ntiles;   // 8x32 output tiles
    int PH, PW;                     // LDS patch extent in padded pixels
    Epilogue ep;                    // forward: elementwise tail before the rounding
};

struct ThinDgradParams {
    const __half* G;     // upstream gradient [N][Ho][Wo][K]
    const __half* WT;    // filter as [C][R][S][K]
    __half* DX;          // [N][H][W][C]
    int N, H, W, C, K, R, S;
    int sh, sw, ph, pw, dh, dw, Ho, Wo;
    int nclasses;
    int class_block_start[17];
    Epilogue ep;
};

struct ThinDgradMfmaParams {
    const __half* G;     // upstream gradient [N][Ho][Wo][K]
    const __half* Wm;    // merged filter [RP*SP][K/8][16 slots][8]
    __half* DX;          // [N][H][W][C]
    int N, H, W, C, K, R, S;
    int sh, sw, ph, pw, dh, dw, Ho, Wo;
    int ohmin, owmin, RP, SP;   // window of dy displacements over all parity classes
    int tiles_i, tiles_j;       // 8x32 macro-pixel tiles
    Epilogue ep;
};

bool thin_dgrad_mfma_supported(const Geom& g);
size_t thin_dgrad_mfma_workspace_bytes(const Geom& g);
hipError_t launch_thin_dgrad_mfma(const Geom& g, const __half* dy, const __half* w, __half* dx, void* ws,
                                  hipStream_t st, const Epilogue& ep = no_epilogue());

bool thin_supported(const Geom& g);
size_t thin_dgrad_lds_bytes(const Geom& g);
hipError_t launch_thin_dgrad(const Geom& g, const __half* dy, const __half* wT, __half* dx, hipStream_t st,
                             const Epilogue& ep = no_epilogue());
size_t thin_packed_filter_bytes(const Geom& g);
size_t thin_wgrad_partial_bytes(const Geom& g);
hipError_t launch_thin_fwd(const Geom& g, const __half* x, const __half* w, __half* y, void* ws, hipStream_t st,
                           const Epilogue& ep = no_epilogue());
hipError_t launch_thin_wgrad(const Geom& g, const __half* x, const __half* dy, float* dw, void* ws, hipStream_t st);

}  // namespace sdconv
