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
//
#pragma once
#include "common.h"
#include "igemm.h"

namespace sdconv {

// With an elementwise tail (P.ep) the strip holds the fp32 accumulators instead, and scale,
// bias, shortcut, ReLU and mask are applied after the read-back, where a lane owns 8 consecutive
// channels of one pixel: the shortcut / mask tensors are read with the same 16-byte row-
// contiguous accesses as the result is written, and the result is rounded to binary16 once.
//
// The strip is sized for the fp32 form (the plain form uses the first half of each row).
template <int WN, int MF = 32> constexpr int epilogue_strip_bytes() { return MF * (WN * 4 + 16); }

// Lanes of one wave hand data to each other through the strip.  The hardware completes the LDS
// operations of a wave in order, but to the compiler the lanes are independent threads: without
// this it may move the writes of lanes that skip the read-back (more lanes than strip chunks)
// past the reads of the others.  No instruction is emitted for it.
__device__ __forceinline__ void strip_handover()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// acc[a][b]: block (rows b*MF.., columns a*MF..) of the wave's WM x WN sub-tile.
// strip: this wave's private LDS area of epilogue_strip_bytes<WN, MF>() bytes; the caller has
// made sure (workgroup barrier) that nobody still reads what the strip overwrites.
// pix_of(r): destination pixel index (n*Hd + h)*Wd + w of row r of the wave's sub-tile, or a
// negative value for rows that have no destination.  col_base: first destination channel.
// MF = 32: accumulators of v_mfma_f32_32x32x16_f16 blocks (16 floats per lane: row lane%32,
// columns 8q + 4*(lane/32) + j); MF = 16: of v_mfma_f32_16x16x32_f16 blocks (4 floats per lane:
// row lane%16, columns 4*(lane/16) + j).  Both as produced by mfma(B fragment, A fragment).
// TAIL: compiled with the elementwise tail (P.ep); the kernels are instantiated both ways so that
// the plain passes keep the registers (and the occupancy) they have without it.
template <int FM, int FN, int MF = 32, bool TAIL = false, typename Acc, typename PixOf>
__device__ __forceinline__ void store_rows_via_lds(Acc (&acc)[FN][FM], unsigned char* strip, int lane,
                                                   int col_base, const IgemmParams& P, PixOf pix_of)
{
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    typedef _Float16 h8 __attribute__((ext_vector_type(8)));
    typedef float f4 __attribute__((ext_vector_type(4)));
    constexpr int WN = FN * MF;
    constexpr int CW = WN / 8;                      // 8-channel chunks per strip row
    constexpr int RPI = 64 / CW;                    // strip rows one store instruction covers
    static_assert(MF % RPI == 0 || RPI % MF == 0, "strip rows per instruction");
    const int lrow = lane & (MF - 1), lhi = lane / MF;
    const int srow = lane / CW, schunk = lane % CW;
    const int col = col_base + schunk * 8;          // first of this lane's 8 destination channels

    if constexpr (!TAIL) {
        constexpr int PITCH = WN * 2 + 16;
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
                    const int scol = (MF == 32) ? a * 32 + 8 * q + 4 * lhi : a * 16 + 4 * lhi;
                    *reinterpret_cast<h4*>(strip + lrow * PITCH + scol * 2) = h;
                }
            }
            // the strip is private to the wave, and LDS operations of one wave complete in order
            strip_handover();
#pragma unroll
            for (int j = 0; j < (MF + RPI - 1) / RPI; ++j) {
                const int r = j * RPI + srow;
                if (RPI <= MF || r < MF) {              // (there may be more lanes than strip chunks)
                    h8 v = *reinterpret_cast<const h8*>(strip + r * PITCH + schunk * 16);
                    const long pix = pix_of(b * MF + r);
                    // streaming store: the result is not read again by this kernel, and keeping it out
                    // of the way of the operand lines in L2 is worth 1.6 % of the detector step
                    if (pix >= 0 && col < P.Cd) __builtin_nontemporal_store(v, reinterpret_cast<h8*>(P.D + pix * P.Cd + col));
                }
            }
            strip_handover();
        }
    } else {
    // ---- with the elementwise tail: fp32 strip ------------------------------------------------
    constexpr int PITCH = WN * 4 + 16;
    constexpr int NJ = (MF + RPI - 1) / RPI;        // read-back instructions per block row
    const Epilogue& E = P.ep;
    const bool live = col < P.Cd;                   // Cd is a multiple of 8 on this route: all 8 or none
    f4 sc0 = {1.f, 1.f, 1.f, 1.f}, sc1 = sc0, bi0 = {0.f, 0.f, 0.f, 0.f}, bi1 = bi0;
    if (live && E.scale) {
        sc0 = *reinterpret_cast<const f4*>(E.scale + col);
        sc1 = *reinterpret_cast<const f4*>(E.scale + col + 4);
    }
    if (live && E.bias) {
        bi0 = *reinterpret_cast<const f4*>(E.bias + col);
        bi1 = *reinterpret_cast<const f4*>(E.bias + col + 4);
    }
    // Destination offsets of everything this lane will store, and the shortcut (or, without
    // one, the mask) values that go with them: all loads are sent before the first strip is
    // written, so their latency passes behind the LDS work instead of once per block row.
    const _Float16* aux = reinterpret_cast<const _Float16*>(E.residual ? E.residual : E.mask);
    int off[FM][NJ];
    h8 pre[FM][NJ];
#pragma unroll
    for (int b = 0; b < FM; ++b)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int r = j * RPI + srow;
            const bool mine = RPI <= MF || r < MF;  // (there may be more lanes than strip chunks)
            const long pix = (mine && live) ? pix_of(b * MF + r) : -1;
            off[b][j] = pix >= 0 ? (int)(pix * P.Cd + col) : -1;
            if (aux && off[b][j] >= 0) pre[b][j] = *reinterpret_cast<const h8*>(aux + off[b][j]);
        }
#pragma unroll
    for (int b = 0; b < FM; ++b) {
#pragma unroll
        for (int a = 0; a < FN; ++a) {
#pragma unroll
            for (int q = 0; q < (MF == 32 ? 4 : 1); ++q) {
                f4 f;
                f[0] = acc[a][b][4 * q + 0];
                f[1] = acc[a][b][4 * q + 1];
                f[2] = acc[a][b][4 * q + 2];
                f[3] = acc[a][b][4 * q + 3];
                const int scol = (MF == 32) ? a * 32 + 8 * q + 4 * lhi : a * 16 + 4 * lhi;
                *reinterpret_cast<f4*>(strip + lrow * PITCH + scol * 4) = f;
            }
        }
        strip_handover();
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int r = j * RPI + srow;
            if (off[b][j] < 0) continue;            // (such a lane reads nothing it would need)
            f4 v0 = *reinterpret_cast<const f4*>(strip + r * PITCH + schunk * 32);
            f4 v1 = *reinterpret_cast<const f4*>(strip + r * PITCH + schunk * 32 + 16);
            float v[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[e] = v0[e] * sc0[e] + bi0[e];
                v[4 + e] = v1[e] * sc1[e] + bi1[e];
            }
            if (E.residual) {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] += (float)pre[b][j][e];
            }
            if (E.relu) {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
            }
            if (E.mask) {
                h8 mm = pre[b][j];
                if (E.residual) mm = *reinterpret_cast<const h8*>(reinterpret_cast<const _Float16*>(E.mask) + off[b][j]);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = (float)mm[e] > 0.f ? v[e] : 0.f;
            }
            h8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (_Float16)v[e];
            __builtin_nontemporal_store(o, reinterpret_cast<h8*>(P.D + off[b][j]));
        }
        strip_handover();
    }
    }
}

// A data-gradient tile of a stride-parity class that no filter tap reaches is all zeros: written
// directly, 16 bytes per lane on consecutive chunks of a pixel row, without tables or strips.
// Rows m_base .. m_base + WM - 1 and columns col_base .. col_base + WN - 1 of the class's GEMM.
template <int WM, int WN>
__device__ __forceinline__ void store_zero_subtile(int lane, int m_base, int col_base, int Mcls, const IgemmParams& P,
                                                   int Hi, int Wj, int eh, int ew, int ca, int cb)
{
    typedef _Float16 h8 __attribute__((ext_vector_type(8)));
    constexpr int CW = WN / 8, RPI = 64 / CW;      // lanes per row, rows per store instruction
    static_assert(64 % CW == 0, "whole rows per instruction");
    const int srow = lane / CW, col = col_base + (lane % CW) * 8;
    const h8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    if (col >= P.Cd) return;
    for (int r = srow; r < WM; r += RPI) {
        const int m = m_base + r;
        if (m >= Mcls) break;
        const int n = m / (Hi * Wj);
        const int rem = m - n * (Hi * Wj);
        const int i = rem / Wj, jj = rem - i * Wj;
        const long pix = ((long)n * P.Hd + (i * eh + ca)) * P.Wd + (jj * ew + cb);
        __builtin_nontemporal_store(z, reinterpret_cast<h8*>(P.D + pix * P.Cd + col));
    }
}

// Rows are GEMM rows m_base.. of an implicit-GEMM tile (pixels of one stride-parity class in
// (n, i, j) order; eh/ew/ca/cb place class pixel (i, j) at (i*eh + ca, j*ew + cb)).
template <int FM, int FN, int MF = 32, bool TAIL = false, typename Acc>
__device__ __forceinline__ void store_tile_via_lds(Acc (&acc)[FN][FM], unsigned char* strip, int lane,
                                                   int m_base, int col_base, int Mcls, const IgemmParams& P,
                                                   int Hi, int Wj, int eh, int ew, int ca, int cb)
{
    const bool linear = (eh == 1 && ew == 1);       // destination pixel index == GEMM row index
    store_rows_via_lds<FM, FN, MF, TAIL>(acc, strip, lane, col_base, P, [&](int r) -> long {
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
