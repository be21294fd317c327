// The "write" step of the depth stream (paper section 2.2): after a layer has run the
// operator, its key-value pair is appended to the depth stream so that later layers can
// read it.  With the position-major cache layout [B, Hk, T, depth_alloc, d] that is a
// strided copy: row (b, g, t) of the layer's K / V [B, Hk, T, d] becomes slot `slot` of
// position (b, g, t).  Bound by HBM bandwidth (every byte is read once and written once);
// 16 bytes per lane, so a wave moves whole rows and the stores are full 128-byte lines.
#include "moda_launch.h"

namespace moda {

constexpr int kAppendPerThread = 2;  // 16-byte chunks of K (and of V) per thread, all loaded before any store

__global__ __launch_bounds__(256) void moda_depth_append_kernel(const char* __restrict__ K, const char* __restrict__ V,
                                                                char* __restrict__ Kd, char* __restrict__ Vd,
                                                                long long n_chunks, int chunks_per_row,
                                                                int depth_alloc, int slot) {
  // chunk i of this thread: (block * kAppendPerThread + u) * 256 + thread, so that a wave's
  // accesses stay contiguous
  const long long base = (long long)blockIdx.x * kAppendPerThread * 256 + threadIdx.x;
  u32x4 kv[kAppendPerThread], vv[kAppendPerThread];
#pragma unroll
  for (int u = 0; u < kAppendPerThread; ++u) {
    const long long i = base + u * 256;
    if (i < n_chunks) {
      // (ordinary loads: the layer's K / V have just been read by its attention and are served
      //  from the caches where they still are; the stores are non-temporal, the cache is not
      //  read again before the next layer)
      kv[u] = *(const u32x4*)(K + (size_t)i * 16);
      vv[u] = *(const u32x4*)(V + (size_t)i * 16);
    }
  }
#pragma unroll
  for (int u = 0; u < kAppendPerThread; ++u) {
    const long long i = base + u * 256;
    if (i < n_chunks) {
      const long long row = i / chunks_per_row;
      const int c = (int)(i - row * chunks_per_row);
      const size_t dst = ((size_t)(row * depth_alloc + slot) * chunks_per_row + c) * 16;
      __builtin_nontemporal_store(kv[u], (u32x4*)(Kd + dst));
      __builtin_nontemporal_store(vv[u], (u32x4*)(Vd + dst));
    }
  }
}

hipError_t launch_depth_append(const void* K, const void* V, void* Kdepth, void* Vdepth, long long rows,
                               int row_bytes, int depth_alloc, int slot, hipStream_t stream) {
  if (row_bytes % 16 != 0) return hipErrorInvalidValue;
  const int cpr = row_bytes / 16;
  const long long n_chunks = rows * cpr;
  const long long blocks = (n_chunks + 256 * kAppendPerThread - 1) / (256 * kAppendPerThread);
  if (!grid_ok(blocks)) return kGridTooLarge;
  return launch_kernel(moda_depth_append_kernel, dim3((unsigned)blocks), dim3(256), stream, (const char*)K,
                       (const char*)V, (char*)Kdepth, (char*)Vdepth, n_chunks, cpr, depth_alloc, slot);
}

}  // namespace moda
