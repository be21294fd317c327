// Shared device-side types and small helpers for the libmoda HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moda {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Kernel arguments of the forward pass.  Pointers are device pointers; layouts
// as documented in include/moda.h.
struct FwdParams {
  const void* Q;
  const void* Kseq;
  const void* Vseq;
  const void* Kdepth;
  const void* Vdepth;
  void* O;
  float* LSE;
  int B, Hq, Hk, T;
  int depth_alloc, depth_count;
  int causal;
  float scale;       // softmax scale (natural units)
  float scale_log2;  // scale * log2(e): logits are exponentiated with exp2
  int n_qtiles;      // tiles along the sequence (bf16 kernel: see heads_per_tile)
  int heads_per_tile;  // bf16 kernel: query heads of one group that share a tile (divides Hq/Hk and the waves)
  int head_group;      // bf16 kernel: heads that one die walks together, tile by tile (0: all its heads)
  int depth_mfma;      // bf16 kernel: depth slots on the matrix pipe (1) or on the vector ALUs (0)
  unsigned depth_magic;  // bf16 kernel: floor(2^32 / depth_count) + 1, so that umulhi(k, magic) = k / depth_count
};

// Kernel arguments of the backward pass (bf16; Hq / Hk query heads share a key/value head).
struct BwdParams {
  const void* Q;
  const void* Kseq;
  const void* Vseq;
  const void* Kdepth;
  const void* Vdepth;
  const void* O;
  const float* LSE;
  const void* dO;
  void* dQ;
  void* dKseq;
  void* dVseq;
  void* dKdepth;
  void* dVdepth;
  float* rowstat;  // workspace: (LSE_t * log2(e), <dO_t, O_t>) per row, [B, Hq, T, 2]
  float* dq_depth;  // workspace: the depth slots' share of dQ, fp32, not yet scaled, [B, Hq, T, d]
  int B, Hq, Hk, T;
  int depth_alloc, depth_count;
  int causal;
  float scale;
  float scale_log2;
  int head_group;  // heads that one die walks together, tile by tile (see head_blocked_id)
};

// Workgroup id -> (head index, tile position in the walking order).  Ids are dealt round-robin
// to the 8 dies (each with its own L2).  With `n_heads` a multiple of 8, die x takes the heads
// x, x + 8, x + 16, ... `group` AT A TIME, each with all its `n_tiles` tiles, instead of a tile
// of every head at a time: the workgroups that run together on a die then stream the K/V (or
// Q/dO) of a few heads, which its L2 holds, and not of n_heads / 8.
__device__ __forceinline__ void head_blocked_id(int id, int n_heads, int n_tiles, int& head, int& tile,
                                                int group = 1) {
  if (group > 0 && n_heads % (8 * group) == 0) {
    const int die = id & 7, r = id >> 3;
    const int per_group = group * n_tiles;
    const int grp = r / per_group, w = r % per_group;
    tile = w / group;
    head = (grp * group + w % group) * 8 + die;
  } else {
    head = id % n_heads;
    tile = id / n_heads;
  }
}

// Value held by lane (l ^ 32) of the same wave.
__device__ __forceinline__ float partner32(float x) {
  int xi = __builtin_bit_cast(int, x);
  auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  // lanes < 32 find the partner's value in r[1], lanes >= 32 in r[0]
  int other = (threadIdx.x & 32) ? r[0] : r[1];
  return __builtin_bit_cast(float, other);
}

// max / sum over the lane pair (l, l ^ 32); symmetric, so no lane select is needed.
__device__ __forceinline__ float pair_max(float x) {
  int xi = __builtin_bit_cast(int, x);
  auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return fmaxf(__builtin_bit_cast(float, (int)r[0]), __builtin_bit_cast(float, (int)r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  int xi = __builtin_bit_cast(int, x);
  auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return __builtin_bit_cast(float, (int)r[0]) + __builtin_bit_cast(float, (int)r[1]);
}

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}
// Sum over aligned groups of LANES (8 or 16) adjacent lanes; every lane gets the result.
template <int LANES>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_mov<0xB1>(x);   // quad_perm [1,0,3,2]
  x += dpp_mov<0x4E>(x);   // quad_perm [2,3,0,1]
  x += dpp_mov<0x141>(x);  // row_half_mirror: lane i <-> 7 - i
  if (LANES == 16) x += dpp_mov<0x140>(x);  // row_mirror: lane i <-> 15 - i
  return x;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Two fp32 -> packed bf16 (round to nearest even), low half = a.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) {
  return __builtin_bit_cast(float, u & 0xffff0000u);
}
// <a, b> over two packed bf16 pairs, accumulated into c in fp32.
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a),
                                         __builtin_bit_cast(bf16x2, b), c, false);
}

}  // namespace moda
