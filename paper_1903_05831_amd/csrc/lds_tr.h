// Tiles kept in LDS as they sit in memory, [contraction row][column] in fp16, and read into
// MFMA fragments with the transposing LDS read.
//
// ds_read_b64_tr_b16 works on groups of 16 lanes: lane 4i+j of a group supplies the address of
// row i, columns 4j..4j+3 (8 bytes) of a 4 x 16 block, and lane n of the group receives column
// n of the four rows.  Two such reads (rows +0..3 and +4..7) give a lane the eight consecutive
// contraction values of its column that v_mfma_f32_32x32x16_f16 wants.
//
// The four rows of a block are a row pitch apart, i.e. on the same banks for any pitch that is
// a multiple of 256 bytes: 64-byte granules of a row are therefore XOR-swizzled with the row
// number.  The 16x16x32 fragments read only 32 bytes of a row per instruction, from rows r..r+3
// and r+8..r+11 in the same half of the wave, so the two 32-byte halves of a granule are swapped
// in rows whose bit 3 is set (without it those reads are two-way bank conflicts: 20 % of the
// weight-gradient kernel's cycles).  The LDS-DMA loads write LDS linearly, so the swizzle is
// applied on the global side, by choosing which 16-byte chunk a lane fetches (swizzled_chunk).
#pragma once
#include <hip/hip_runtime.h>

namespace sdconv {

typedef _Float16 tr_half4 __attribute__((ext_vector_type(4)));
typedef _Float16 tr_half8 __attribute__((ext_vector_type(8)));
typedef short tr_short4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ tr_half4 lds_read_tr16(const unsigned char* p)
{
    typedef __attribute__((address_space(3))) tr_short4* lds_ptr;
    tr_short4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    return __builtin_bit_cast(tr_half4, v);
}

// granule mask of a [rows][BW halves] tile
template <int BW> constexpr int tr_gmask() { return (BW * 2 >= 256) ? 3 : (BW * 2 / 64 - 1); }

// Byte offset of (row, col half-index) in a [rows][BW halves] tile with swizzled granules.
template <int BW>
__device__ __forceinline__ int sw_off(int row, int col)
{
    constexpr int pitch = BW * 2;
    int byte = col * 2;
    int gran = (byte >> 6) ^ (row & tr_gmask<BW>());
    return row * pitch + (gran << 6) + ((byte & 63) ^ (((row >> 3) & 1) << 5));
}

// Logical 16-byte chunk of row `row` that the lane filling physical chunk slot `pc` fetches.
template <int BW>
__device__ __forceinline__ int swizzled_chunk(int row, int pc)
{
    return (((pc >> 2) ^ (row & tr_gmask<BW>())) << 2) | ((pc & 3) ^ (((row >> 3) & 1) << 1));
}

// Fragment of the 32 columns starting at col0 (a multiple of 32), contraction rows
// row0 .. row0+15 (lanes 0-31 get rows +0..7, lanes 32-63 rows +8..15), of the tile at `tile`.
template <int BW>
__device__ __forceinline__ tr_half8 lds_frag_tr(const unsigned char* tile, int row0, int col0, int lane)
{
    const int grp = lane >> 4, gl = lane & 15;
    const int row = row0 + 8 * (grp >> 1) + (gl >> 2);
    const int col = col0 + 16 * (grp & 1) + 4 * (gl & 3);
    tr_half4 lo = lds_read_tr16(tile + sw_off<BW>(row, col));
    tr_half4 hi = lds_read_tr16(tile + sw_off<BW>(row + 4, col));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Same for v_mfma_f32_16x16x32_f16: fragment of the 16 columns starting at col0 (a multiple of
// 16), contraction rows row0 .. row0+31 (lane group g = lane/16 gets rows +8g..8g+7).
template <int BW>
__device__ __forceinline__ tr_half8 lds_frag_tr_16(const unsigned char* tile, int row0, int col0, int lane)
{
    const int grp = lane >> 4, gl = lane & 15;
    const int row = row0 + 8 * grp + (gl >> 2);
    const int col = col0 + 4 * (gl & 3);
    tr_half4 lo = lds_read_tr16(tile + sw_off<BW>(row, col));
    tr_half4 hi = lds_read_tr16(tile + sw_off<BW>(row + 4, col));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

}  // namespace sdconv
