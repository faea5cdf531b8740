// Epilogue shared by the LDS-DMA implicit-GEMM kernels: fp32 accumulators -> fp16 (nearest
// even) -> NHWC destination, transposed through LDS so that the global stores are 16 bytes per
// lane on consecutive chunks of a pixel row.
//
// A lane's accumulators of one 32x32 MFMA block (computed as B x A, i.e. transposed) are 16
// columns of ONE pixel row, in four groups of four: stored directly they become 8-byte pieces
// scattered over 32 rows, sixteen partial writes per 128-byte line.  Here each wave parks
// 32 rows x WN columns in a private LDS strip (row pitch padded by 16 bytes against bank
// conflicts) and reads it back with consecutive lanes on consecutive 16-byte chunks of a row,
// so every store instruction writes whole 64/128-byte row segments.
#pragma once
#include "common.h"
#include "igemm.h"

namespace sdconv {

template <int WN, int MF = 32> constexpr int epilogue_strip_bytes() { return MF * (WN * 2 + 16); }

// acc[a][b]: block (rows b*32.., columns a*32..) of the wave's WM x WN sub-tile.
// strip: this wave's private LDS area of epilogue_strip_bytes<WN>() bytes; the caller has made
// sure (workgroup barrier) that nobody still reads what the strip overwrites.
// pix_of(r): destination pixel index (n*Hd + h)*Wd + w of row r of the wave's sub-tile, or a
// negative value for rows that have no destination.  col_base: first destination channel.
// MF = 32: accumulators of v_mfma_f32_32x32x16_f16 blocks (16 floats per lane: row lane%32,
// columns 8q + 4*(lane/32) + j); MF = 16: of v_mfma_f32_16x16x32_f16 blocks (4 floats per lane:
// row lane%16, columns 4*(lane/16) + j).  Both as produced by mfma(B fragment, A fragment).
template <int FM, int FN, int MF = 32, typename Acc, typename PixOf>
__device__ __forceinline__ void store_rows_via_lds(Acc (&acc)[FN][FM], unsigned char* strip, int lane,
                                                   int col_base, const IgemmParams& P, PixOf pix_of)
{
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    typedef _Float16 h8 __attribute__((ext_vector_type(8)));
    constexpr int WN = FN * MF;
    constexpr int CW = WN / 8;                      // 16-byte chunks per strip row
    constexpr int RPI = 64 / CW;                    // strip rows one store instruction covers
    constexpr int PITCH = WN * 2 + 16;
    static_assert(MF % RPI == 0 || RPI % MF == 0, "strip rows per instruction");
    const int lrow = lane & (MF - 1), lhi = lane / MF;
    const int srow = lane / CW, schunk = lane % CW;
#pragma unroll
    for (int b = 0; b < FM; ++b) {
#pragma unroll
        for (int a = 0; a < FN; ++a) {
#pragma unroll
            for (int q = 0; q < (MF == 32 ? 4 : 1); ++q) {
                h4 h;
                h[0] = (_Float16)acc[a][b][4 * q + 0];
                h[1] = (_Float16)acc[a][b][4 * q + 1];
                h[2] = (_Float16)acc[a][b][4 * q + 2];
                h[3] = (_Float16)acc[a][b][4 * q + 3];
                const int col = (MF == 32) ? a * 32 + 8 * q + 4 * lhi : a * 16 + 4 * lhi;
                *reinterpret_cast<h4*>(strip + lrow * PITCH + col * 2) = h;
            }
        }
        // the strip is private to the wave, and LDS operations of one wave complete in order
#pragma unroll
        for (int j = 0; j < (MF + RPI - 1) / RPI; ++j) {
            const int r = j * RPI + srow;
            if (RPI > MF && r >= MF) continue;      // more lanes than strip chunks
            h8 v = *reinterpret_cast<const h8*>(strip + r * PITCH + schunk * 16);
            const int col = col_base + schunk * 8;
            const long pix = pix_of(b * MF + r);
            if (pix >= 0 && col < P.Cd) *reinterpret_cast<h8*>(P.D + pix * P.Cd + col) = v;
        }
    }
}

// Rows are GEMM rows m_base.. of an implicit-GEMM tile (pixels of one stride-parity class in
// (n, i, j) order; eh/ew/ca/cb place class pixel (i, j) at (i*eh + ca, j*ew + cb)).
template <int FM, int FN, int MF = 32, typename Acc>
__device__ __forceinline__ void store_tile_via_lds(Acc (&acc)[FN][FM], unsigned char* strip, int lane,
                                                   int m_base, int col_base, int Mcls, const IgemmParams& P,
                                                   int Hi, int Wj, int eh, int ew, int ca, int cb)
{
    const bool linear = (eh == 1 && ew == 1);       // destination pixel index == GEMM row index
    store_rows_via_lds<FM, FN, MF>(acc, strip, lane, col_base, P, [&](int r) -> long {
        const int m = m_base + r;
        if (m >= Mcls) return -1;
        if (linear) return m;
        int n = m / (Hi * Wj);
        int rem = m - n * (Hi * Wj);
        int i = rem / Wj, jj = rem - i * Wj;
        return ((long)n * P.Hd + (i * eh + ca)) * P.Wd + (jj * ew + cb);
    });
}

}  // namespace sdconv
