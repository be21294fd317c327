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
//   d = 128 (16 chunks, a row = all banks):      swz(r) = ((r & 3) << 2) | ((r >> 2) & 3);
//   d = 64  ( 8 chunks, two rows = all banks):   swz(r) = (((r >> 1) & 1) << 2) | ((r >> 2) & 3).
// Both meet both conditions (measured: bank-conflict cycles 43-66 % of the LDS cycles with the
// pair permutation used before, 0 with these).
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
    return D == 128 ? (((r & 3) << 2) | ((r >> 2) & 3)) : ((((r >> 1) & 1) << 2) | ((r >> 2) & 3));
  }
  // byte offset of the 16-byte chunk c of row r
  __device__ static __forceinline__ int off(int r, int c) { return r * kRowBytes + ((c ^ swz(r)) << 4); }
};

// x ^ c, evaluated where it is written.  The compiler would otherwise precompute one address
// per fragment outside the loops and keep them all in registers; the kernels that use these
// tiles have none to spare, the addresses end up in scratch memory, and every reload from
// scratch waits for ALL earlier memory operations, the tile copies in flight included.
__device__ __forceinline__ int xor_here(int x, int c) {
  if (c == 0) return x;
  int r;
  asm volatile("v_xor_b32 %0, %1, %2" : "=v"(r) : "s"(c), "v"(x));
  return r;
}

// Per-lane fragment addresses inside a tile: three registers and constants.  Channel step st
// of a row fragment and channel block db of a transposed fragment only flip bits 5..7 of the
// chunk field (an XOR, because the chunk index is permuted by an XOR); row blocks are
// immediates.
template <int D>
struct FragAddr {
  using Tl = Tile<D>;
  int row;  // chunk `hi` of row l32 (st = 0, rb = 0)
  int tr;   // first read of transposed fragment (ks = 0, db = 0)
  int tr8;  // second read: the rows 8 further on
  __device__ __forceinline__ void init(int lane) {
    const int l32 = lane & 31, hi = lane >> 5;
    row = Tl::off(l32, hi);
    const int rr = hi * 4 + ((lane & 15) >> 2);
    const int grp = (lane >> 4) & 1;
    // this lane's 8 bytes: piece (lane & 3) of the two chunks of a 16-channel block (chunks are
    // permuted one by one, so the two need not be adjacent)
    const int ch = grp * 2 + ((lane & 3) >> 1);
    tr = Tl::off(rr, ch) + (lane & 1) * 8;
    tr8 = Tl::off(rr + 8, ch) + (lane & 1) * 8;
  }
  // Addresses are formed as  xor_here(base, constant) + immediate:  `base` = one of the three
  // registers plus the LDS address of a tile (a multiple of 256, so that the XOR, which only
  // touches bits 5..7, commutes with that addition), the immediate = row block, and - for the
  // second tile of a stage, which sits kBytes after the first - the tile.  One XOR thus serves
  // the fragments at the same place of both tiles of a stage.
  // row fragment: rows rb*32 .. rb*32+31 of the tile `tile_off` bytes after the one in `xbase`
  __device__ static __forceinline__ bf16x8 row_frag(unsigned xbase, int rb, int tile_off) {
    return *(const bf16x8 __attribute__((address_space(3)))*)(size_t)(xbase + rb * 32 * Tl::kRowBytes + tile_off);
  }
  // transposed fragment: rows ks*16 .. ks*16+15 (x0: first read, x8: the rows 8 further on)
  __device__ static __forceinline__ bf16x8 tr_frag(unsigned x0, unsigned x8, int ks, int tile_off) {
    const unsigned o = ks * 16 * Tl::kRowBytes + tile_off;
    s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(size_t)(x0 + o));
    s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(size_t)(x8 + o));
    s16x8 v01 = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v01);
  }
};

// 16 bytes per lane, global -> LDS without register staging: lane i's bytes land at
// lds_addr + 16 i.  The source is a raw buffer (base, size in bytes): lanes whose offset falls
// outside it fetch nothing and write zeros, so rows past the end of the matrix need no
// clamping (callers mask them).  Completion is awaited with wait_copies() before the barrier
// that publishes the tile.
__device__ __forceinline__ i32x4 make_tile_buffer(const void* base, unsigned bytes) {
  const unsigned long long b = (unsigned long long)base;
  i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)(b & 0xffffffffu));
  r[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((b >> 32) & 0xffffu));  // stride 0
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;  // 32-bit untyped data
  return r;
}
__device__ __forceinline__ void tile_copy16(const i32x4& rsrc, int voff, int soff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(__builtin_amdgcn_readfirstlane((int)lds_addr)), "v"(voff), "s"(rsrc),
                 "s"(__builtin_amdgcn_readfirstlane(soff))
               : "memory");
}
__device__ __forceinline__ void wait_copies() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Copies rows [row0, row0+64) of a [n_rows, D] bf16 matrix (behind `rsrc`) into a tile, 1 KB
// pieces (1024 / row bytes rows each), piece q by copy instruction q % kInstPerWave of wave
// q / kInstPerWave.  The chunk permutation is applied by choosing which global chunk a lane
// fetches.  ONE per-lane register serves all pieces: the permutation of piece q differs from
// piece 0's by a constant XOR that only depends on the parity of q (see swz), and everything
// else is wave-uniform.  (With one offset register per piece, the compiler spilled them, and a
// reload from scratch memory in front of every copy instruction waits for ALL earlier memory
// operations, the previous copy included: the copies of a tile then ran one memory round trip
// after the other.)
template <int D, int NW = 4>
struct TileLoader {
  static constexpr int kRowsPerInst = 64 / Tile<D>::kChunks;
  static constexpr int kInstPerWave = 64 / kRowsPerInst / NW;
  static_assert(kInstPerWave >= 1, "every wave copies part of every tile");
  // byte XOR between the offsets of piece q and piece 0: swz of the piece's first row
  // (d = 128: 4 rows per piece, swz(4q) = q & 3; d = 64: 8 rows per piece, swz(8q) = (q & 1) << 1)
  __device__ __host__ static constexpr int piece_xor(int q) { return (D == 128 ? (q & 3) : ((q & 1) << 1)) << 4; }
  static_assert(kInstPerWave == 1 || kInstPerWave == 2 || kInstPerWave == 4,
                "piece_xor(wave * kInstPerWave + i) = piece_xor(wave * kInstPerWave) ^ piece_xor(i)");
  int goff;
  int wave;
  __device__ __forceinline__ void init(int wave_, int lane) {
    wave = wave_;
    const int j = lane / Tile<D>::kChunks;   // row inside the piece
    const int pc = lane % Tile<D>::kChunks;  // chunk position this lane fills
    goff = j * Tile<D>::kRowBytes + ((pc ^ Tile<D>::swz(j)) << 4);
    goff ^= piece_xor(wave * kInstPerWave);  // the wave's first piece; piece i of the wave: ^ piece_xor(i)
  }
  __device__ __forceinline__ void issue(const i32x4& rsrc, int row0, unsigned lds_addr) const {
#pragma unroll
    for (int i = 0; i < kInstPerWave; ++i) {
      const int q = wave * kInstPerWave + i;
      const int voff = xor_here(goff, piece_xor(i));
      tile_copy16(rsrc, voff, row0 * Tile<D>::kRowBytes + q * 1024, lds_addr + q * 1024);
    }
  }
};

// Eight fp32 -> one MFMA operand of packed bf16 (round to nearest even).
__device__ __forceinline__ bf16x8 pack8(const float (&x)[8]) {
  u32x4 t = {pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7])};
  return __builtin_bit_cast(bf16x8, t);
}

__device__ __forceinline__ f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

}  // namespace moda
