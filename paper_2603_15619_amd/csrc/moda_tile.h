// LDS tile helpers shared by the backward kernels (gfx950).
//
// A tile is 64 rows x D channels of bf16, row-major, with the 16-byte chunks of a row
// permuted by an XOR with a function of the row index: chunk c of row r sits at chunk
// position c ^ swz(r).  For both access patterns used below to touch every LDS bank once
// (64 banks x 4 bytes = 256 bytes per cycle):
//   - a row-fragment read takes the same logical chunk of 16 consecutive rows: swz must
//     give those rows 16 different (half-of-256-bytes, chunk position) places;
//   - a transposing read takes, per cycle, one 64-byte segment (4 chunks) of 4 consecutive
//     rows: swz must send those rows to different 64-byte bank groups, i.e. differ in its
//     bit 2 (and bit 3 at d = 128) among them.
//   d = 64  ( 8 chunks, two rows = all banks): swz(r) = (((r >> 1) & 1) << 2) | ((r >> 2) & 3)
//           meets both (measured: bank-conflict cycles 50-66 % -> 0, kernels 3-13 % faster).
//   d = 128 (16 chunks, a row = all banks): ((r & 3) << 2) | ((r >> 2) & 3) meets both as well,
//           but the rows r and r + 8 of a transposed fragment then differ in their permutation,
//           which costs the dK/dV kernel four more address registers than it has (measured:
//           conflicts 43 % -> 0, yet 1.78 -> 2.03 ms because of spills).  It keeps
//           swz(r) = (r & 7) << 1, a 2-way conflict on both patterns.
// The access patterns:
//   row fragment  (MFMA A operand, M = rows, K = channels): lane l reads 16 bytes of
//                 row (l % 32), channels 16*st + 8*(l/32) .. +7;
//   transposed fragment (MFMA A operand, M = channels, K = rows), built from two
//                 ds_read_b64_tr_b16: within 16 lanes, lane i supplies row (i/4),
//                 8-byte piece (i%4) of a 4-row x 16-channel block and receives
//                 channel i of the 4 rows.  MFMA k-slots 0..7 (lanes < 32) are rows
//                 {0..3, 8..11} of a 16-row group and slots 8..15 (lanes >= 32) rows
//                 {4..7, 12..15}: the order in which a 32x32 accumulator holds its
//                 rows, so that an accumulator (packed to bf16) is directly the B
//                 operand of the product that contracts over those rows.
#pragma once
#include "moda_common.h"

namespace moda {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr;

template <int D>
struct Tile {
  static constexpr int kRows = 64;
  static constexpr int kChunks = D / 8;
  static constexpr int kRowBytes = D * 2;
  static constexpr int kBytes = kRows * kRowBytes;
  static constexpr int kDSteps = D / 16;
  static constexpr int kDBlocks = D / 32;

  __device__ static __forceinline__ int swz(int r) {
    return D == 128 ? ((r & 7) << 1) : ((((r >> 1) & 1) << 2) | ((r >> 2) & 3));
  }
  // byte offset of the 16-byte chunk c of row r
  __device__ static __forceinline__ int off(int r, int c) { return r * kRowBytes + ((c ^ swz(r)) << 4); }
  // row fragment: rows rb*32 .. rb*32+31, channel step st
  __device__ static __forceinline__ bf16x8 row_frag(const unsigned char* tile, int rb, int st, int lane) {
    const int l32 = lane & 31, hi = lane >> 5;
    return *(const bf16x8*)(tile + off(rb * 32 + l32, st * 2 + hi));
  }
  // transposed fragment: rows ks*16 .. ks*16+15, channels db*32 .. db*32+31
  __device__ static __forceinline__ bf16x8 tr_frag(const unsigned char* tile, int ks, int db, int lane) {
    const int hi = lane >> 5;
    const int rr = ks * 16 + hi * 4 + ((lane & 15) >> 2);
    // this lane's 8 bytes: piece (lane & 3) of the two chunks of a 16-channel block.  At
    // d = 128 the permutation keeps the two chunks adjacent and the rows r, r + 8 alike (one
    // address computation serves both); at d = 64 chunks are permuted one by one.
    const unsigned char *a0, *a1;
    if constexpr (D == 128) {
      const int ch = db * 4 + ((lane >> 4) & 1) * 2;
      a0 = tile + off(rr, ch) + (lane & 3) * 8;
      a1 = a0 + 8 * kRowBytes;
    } else {
      const int ch = db * 4 + ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
      a0 = tile + off(rr, ch) + (lane & 1) * 8;
      a1 = tile + off(rr + 8, ch) + (lane & 1) * 8;
    }
    s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)a0);
    s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)a1);
    s16x8 v01 = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v01);
  }
};

// 16 bytes per lane, global -> LDS without register staging: lane i's bytes land at
// lds_addr + 16 i.  Completion is awaited with wait_copies() before the barrier that
// publishes the tile.
__device__ __forceinline__ void tile_copy16(const char* gbase, int voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(gbase)
               : "memory");
}
__device__ __forceinline__ void wait_copies() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Copies rows [row0, row0+64) of a [n_rows, D] bf16 matrix into a tile; rows past
// n_rows re-read the last row (callers mask them).  All NW waves of the workgroup take part.
template <int D, int NW = 4>
struct TileLoader {
  static constexpr int kRowsPerInst = 64 / Tile<D>::kChunks;
  static constexpr int kInstPerWave = 64 / kRowsPerInst / NW;
  static_assert(kInstPerWave >= 1, "every wave copies part of every tile");
  int goff[kInstPerWave];
  int row[kInstPerWave];
  int wave;
  __device__ __forceinline__ void init(int wave_, int lane) {
    wave = wave_;
#pragma unroll
    for (int i = 0; i < kInstPerWave; ++i) {
      const int r = (wave * kInstPerWave + i) * kRowsPerInst + lane / Tile<D>::kChunks;
      const int pc = lane % Tile<D>::kChunks;  // chunk position this lane fills
      const int c = pc ^ Tile<D>::swz(r);
      row[i] = r;
      goff[i] = r * Tile<D>::kRowBytes + c * 16;
    }
  }
  __device__ __forceinline__ void issue(const char* gmat, int row0, int n_rows, unsigned lds_addr) const {
    const char* gt = gmat + (size_t)row0 * Tile<D>::kRowBytes;
    const int valid = n_rows - row0;
#pragma unroll
    for (int i = 0; i < kInstPerWave; ++i) {
      const int r = min(row[i], valid - 1);
      tile_copy16(gt, goff[i] + (r - row[i]) * Tile<D>::kRowBytes,
                  lds_addr + (wave * kInstPerWave + i) * kRowsPerInst * Tile<D>::kRowBytes);
    }
  }
};

__device__ __forceinline__ f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

}  // namespace moda
