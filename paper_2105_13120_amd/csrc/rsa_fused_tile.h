// LDS tile layout shared by the fused RSA kernels: a tile is 64 rows (tokens)
// by 64 bf16 (the head dimension A, or one half of it when A = 128), 8 KiB, with no padding.  Row r occupies
// bytes [128 r, 128 r + 128); inside the row the eight 16-byte chunks are
// permuted: logical chunk cc sits at position cc ^ rot3((r >> 1) & 7), where
// rot3 rotates a 3-bit value right by one.  With 64 four-byte banks this makes
// all three access patterns conflict-free:
//   * the 16-byte stores of the global->LDS copy (a 16-lane phase is 2 rows x 8 chunks),
//   * 16-byte MFMA operand reads along a row (a phase is 16 consecutive rows, one chunk),
//   * 8-byte transpose reads (a 32-lane phase is 4 rows x 4 chunks).
#pragma once
#include "rsa_common.h"

namespace rsa {

constexpr int kTileKeys = 64;
constexpr int kTileBytes = 64 * 64 * 2;

__device__ __forceinline__ int swz_rot(int row) {
  const int t = (row >> 1) & 7;
  return ((t & 1) << 2) | (t >> 1);
}
// byte offset of 16-byte chunk `cc` (elements 8 cc .. 8 cc + 7) of row `row`
__device__ __forceinline__ int tile_off(int row, int cc) {
  return row * 128 + ((cc ^ swz_rot(row)) << 4);
}

// Per-lane byte offsets for the two kinds of MFMA operand fetch from a tile.
struct TileLanes {
  int rows_off[4];     // [dk]
  int cols_off[2][2];  // [db][e8]

  __device__ __forceinline__ explicit TileLanes(int lane) {
    const int col = lane & 31, half = lane >> 5;
#pragma unroll
    for (int dk = 0; dk < 4; ++dk) rows_off[dk] = tile_off(col, dk * 2 + half);
    const int g = lane >> 4, j = lane & 15;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int e8 = 0; e8 < 2; ++e8) {
        const int row = e8 * 8 + half * 4 + (j >> 2);
        const int cc = db * 4 + (g & 1) * 2 + ((j >> 1) & 1);
        cols_off[db][e8] = tile_off(row, cc) + (j & 1) * 8;
      }
  }

  // Operand whose MFMA row/column index runs over tile rows: lane (col, half)
  // gets tile[row_base + col][dk*16 + half*8 .. +8].  row_base: multiple of 32.
  __device__ __forceinline__ bf16x8 read_rows(const unsigned char *tile, int row_base, int dk) const {
    return *reinterpret_cast<const bf16x8 *>(tile + row_base * 128 + rows_off[dk]);
  }

  // The same operand with the k index of slice dk taken in the order read_cols delivers it
  // (element e <-> column dk*16 + (e>>2)*8 + half*4 + (e&3)), for an MFMA whose other operand
  // comes from read_cols.  The row read gives lane (col, 0) columns 0..7 and lane (col, 1)
  // columns 8..15 of the slice; the wanted order is (0..3, 8..11) and (4..7, 12..15), i.e. the
  // upper 8 bytes of the first lane change places with the lower 8 bytes of the second.
  __device__ __forceinline__ bf16x8 read_rows_perm(const unsigned char *tile, int row_base, int dk) const {
    u32x4 w = __builtin_bit_cast(u32x4, read_rows(tile, row_base, dk));
    uint32_t lo0 = w[0], lo1 = w[1], hi0 = w[2], hi1 = w[3];
    permlane32_swap(lo0, hi0);
    permlane32_swap(lo1, hi1);
    const u32x4 r = {lo0, lo1, hi0, hi1};
    return __builtin_bit_cast(bf16x8, r);
  }

  // Operand whose MFMA row index runs over the head dimension and whose k
  // index runs over 16 tile rows: lane (col, half) gets, for e = 0..7,
  //   tile[row_base + (e>>2)*8 + half*4 + (e&3)][db*32 + col],
  // which is the k order in which a 32x32 accumulator holds its rows
  // (elements u*8 .. u*8+7 of lane-half `half`).  row_base: multiple of 16.
  __device__ __forceinline__ bf16x8 read_cols(const unsigned char *tile, int row_base, int db) const {
    const u32x2 lo = lds_read_tr16(tile + row_base * 128 + cols_off[db][0]);
    const u32x2 hi = lds_read_tr16(tile + row_base * 128 + cols_off[db][1]);
    const u32x4 w = {lo[0], lo[1], hi[0], hi[1]};
    return __builtin_bit_cast(bf16x8, w);
  }
};

// Direct global->LDS copy of one 64 x 64 bf16 tile by a work-group of WAVES (4 or 8) waves:
// wave w moves the 16-byte pieces (PER w + j) * 64 + lane, j < PER = 8 / WAVES; the piece at LDS position
// p = 8 row + pc holds logical chunk pc ^ rot(row) of that row, so the tile lands in the
// swizzled layout above.  `g` points at element [0][0] of the tile in global memory
// (rows `ld` elements apart).
// Completion: wait_vmem(), then a barrier.
// A wave's block of 32 output rows x 64 columns, held transposed in two accumulators
// (acc[db]: rows = columns db*32 .. +32 of the output, column = output row), is put into rows
// row_base .. +32 of the wave's own LDS tile as bf16 (times `scale`).
__device__ __forceinline__ void stage_block_T(unsigned char *tile, int row_base, const f32x16 &acc0,
                                              const f32x16 &acc1, float scale, int lane) {
  const int col = lane & 31, half = lane >> 5;
#pragma unroll
  for (int db = 0; db < 2; ++db) {
    const f32x16 &c = db == 0 ? acc0 : acc1;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const u32x2 w = {pack_bf16(c[g * 4 + 0] * scale, c[g * 4 + 1] * scale),
                       pack_bf16(c[g * 4 + 2] * scale, c[g * 4 + 3] * scale)};
      *reinterpret_cast<u32x2 *>(tile + tile_off(row_base + col, db * 4 + g) + half * 8) = w;
    }
  }
}
// ... and rows [first, first + ROWS) of the tile leave for global memory (64 bf16 of each row,
// rows `ld` elements apart) as 16-byte pieces: one wave instruction stores 8 rows of 128 bytes.
// Rows at or beyond rows_valid (counted from row 0 of g) are skipped.
template <int ROWS>
__device__ __forceinline__ void flush_rows(const unsigned char *tile, int first, uint16_t *g,
                                           int64_t rows_valid, int lane, int ld = 64) {
#pragma unroll
  for (int it = 0; it < ROWS / 8; ++it) {
    const int row = it * 8 + (lane >> 3), cc = lane & 7;
    if (row < rows_valid)
      *reinterpret_cast<u32x4 *>(g + (int64_t)row * ld + cc * 8) =
          *reinterpret_cast<const u32x4 *>(tile + tile_off(first + row, cc));
  }
}

template <int WAVES>
struct TileDMAT {
  static constexpr int PER = 8 / WAVES;
  int g_off[PER], l_off[PER];
  // ld: elements between consecutive rows of the tile in global memory (at most 2^24)
  __device__ __forceinline__ TileDMAT(int wave, int lane, int ld) {
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int p = (wave * PER + j) * 64 + lane;
      const int row = p >> 3, cc = (p & 7) ^ swz_rot(row);
      g_off[j] = row * ld + cc * 8;
      l_off[j] = (wave * PER + j) * 1024;
    }
  }
  __device__ __forceinline__ void load(const uint16_t *g, unsigned char *tile) const {
#pragma unroll
    for (int j = 0; j < PER; ++j) lds_dma16(g + g_off[j], tile + l_off[j]);
  }
};
using TileDMA = TileDMAT<4>;

}  // namespace rsa
