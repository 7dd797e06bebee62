// Un-padded, XOR-swizzled LDS tiles for head dims 64 / 128 / 256 / 512 and the LDS transpose read.
//
// A tile is ROWS x D bf16, row-major, 2*D bytes per row, made of 16-byte chunks.  Chunk c of row r is
// stored at chunk position c ^ swz<D>(r).  The swizzle makes all three access patterns used by the
// kernels bank-conflict free on the 64-bank LDS:
//   * 16-byte staging writes (16 lanes = consecutive chunks of a row),
//   * 16-byte MFMA operand reads with the lane on the row axis (16 lanes = 16 consecutive rows, same
//     chunk),
//   * ds_read_b64_tr_b16 transpose reads with the lane on the column axis (16 lanes = 4 consecutive
//     rows x 32 contiguous bytes; the neighbouring 16 lanes read the next 32 bytes of the same rows).
//
// ds_read_b64_tr_b16: within each group of 16 lanes, lane i supplies the address of 4 consecutive
// 16-bit values; viewing the 16 x 4 values as a flat list v[0..63] (lane-major), lane i receives
// v[i], v[16+i], v[32+i], v[48+i].  With lane i pointing at row k0 + i/4, columns d0 + 4*(i%4) .. +3 of
// a row-major tile, lane i therefore receives column d0 + i of rows k0 .. k0+3: a K-indexed MFMA
// operand of the transposed tile without any transposed copy in LDS.
#pragma once
#include "common.h"

namespace dkv {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

template <int D>
__device__ __forceinline__ int swz(int row) {
  static_assert(D == 64 || D == 128 || D == 256 || D == 512, "swizzle defined for 64 / 128 / 256 / 512");
  // (the 512- and 1024-byte rows of head dims 256 and 512 span several bank lines: the chunk index bits from 4 on
  // do not select a bank)
  if (D >= 128) return ((row & 3) << 2) | ((row >> 2) & 3);
  return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
}

// byte offset of chunk `chunk` of row `row` inside a tile
template <int D>
__device__ __forceinline__ int tile_off(int row, int chunk) {
  return row * (2 * D) + ((chunk ^ swz<D>(row)) << 4);
}

// Per-lane byte offset for a transpose read of rows (row_base + (lane%16)/4), columns
// col_base + 16*((lane/16)%2) + 4*(lane%4) .. +3, where row_base is a multiple of 4 given relative to a
// 16-row aligned origin (the swizzle has period 16 rows).
template <int D>
__device__ __forceinline__ int tr_off(int lane, int row_base, int col_base) {
  const int r16 = lane & 15, g = (lane >> 4) & 1;
  const int row = row_base + (r16 >> 2);
  const int col = col_base + g * 16 + (r16 & 3) * 4;
  return tile_off<D>(row, col >> 3) + ((col >> 2) & 1) * 8;
}

// two transpose reads (rows k0..k0+3 and k0+8..k0+11 of the lane's group) -> one MFMA operand
__device__ __forceinline__ bf16x8 tr_pair(const unsigned char* a0, const unsigned char* a1) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(a0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(a1));
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// ---------------------------------------------------------------------------------------------
// Transposed image of a 64-row tile: image row = column index of the source tile (one per head-dim
// value), 128 bytes per image row holding the 64 source rows in "kperm" order (within every group of
// 16 the two middle groups of four are swapped, so the eight contraction indices one MFMA lane needs
// are one contiguous 16-byte chunk).  16-byte chunk c of image row d sits at chunk position
// c ^ ((d / 2) % 8): two image rows share a 256-byte bank line, and the swizzle makes the operand reads
// (16 lanes = 16 consecutive image rows, same chunk) conflict free.  Measured on gfx950, 16-byte reads of
// such an image sustain about 2.5x the bytes per cycle of ds_read_b64_tr_b16 on a row-major tile, so the
// kernels pay the transposition once, at staging time, instead of on every operand read.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int tt_off(int d, int chunk) { return d * 128 + ((chunk ^ ((d >> 1) & 7)) << 4); }

// Store the 4 x 8 block of source rows 4*rq .. 4*rq+3, columns 8*ch .. 8*ch+7 (one 16-byte load per row,
// v[0..3]) into the transposed image: eight 8-byte writes.
__device__ __forceinline__ void store_unit_transposed(unsigned char* img, u32x4 r0, u32x4 r1, u32x4 r2, u32x4 r3,
                                                      int rq, int ch) {
  const int pos4 = kperm4(rq);
  const int coff = (pos4 & 1) * 8;
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    u32x2 lo, hi;
    lo.x = (r0[m] & 0xffffu) | (r1[m] << 16);
    lo.y = (r2[m] & 0xffffu) | (r3[m] << 16);
    hi.x = (r0[m] >> 16) | (r1[m] & 0xffff0000u);
    hi.y = (r2[m] >> 16) | (r3[m] & 0xffff0000u);
    const int d0 = ch * 8 + 2 * m;
    *reinterpret_cast<u32x2*>(img + tt_off(d0, pos4 >> 1) + coff) = lo;
    *reinterpret_cast<u32x2*>(img + tt_off(d0 + 1, pos4 >> 1) + coff) = hi;
  }
}

}  // namespace dkv
