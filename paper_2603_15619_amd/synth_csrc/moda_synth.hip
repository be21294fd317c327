// Seeded synthetic inputs, generated on the device: iid N(0,1) values from a counter-based
// generator (a 64-bit mixing function of (seed, tensor id, element pair index) -> two uniform
// numbers -> Box-Muller), rounded to the requested type.  A library of its own
// (libmoda_synth.so): it holds none of the attention arithmetic and shares no code with libmoda
// or with the CPU checker; both consume the buffers it fills.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

// Finaliser of a well-known 64-bit hash (two multiply-xorshift rounds): every input bit affects
// every output bit.
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x ^= x >> 33;
  x *= 0xff51afd7ed558ccdull;
  x ^= x >> 33;
  x *= 0xc4ceb9fe1a85ec53ull;
  x ^= x >> 33;
  return x;
}

__device__ __forceinline__ uint16_t to_bf16(float f) {  // round to nearest even
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <bool BF16>
__global__ __launch_bounds__(256) void moda_synth_normal_kernel(void* out, unsigned long long n_pairs,
                                                                unsigned long long n, unsigned long long key) {
  const unsigned long long j = (unsigned long long)blockIdx.x * 256 + threadIdx.x;  // pair index
  if (j >= n_pairs) return;
  const uint64_t h = mix64(mix64(key) + j * 0x9e3779b97f4a7c15ull);
  // two uniforms in (0, 1): 24 bits each, centred in their cell so that neither 0 nor 1 occurs
  const float u1 = ((float)(uint32_t)(h >> 40) + 0.5f) * (1.0f / 16777216.0f);
  const float u2 = ((float)(uint32_t)(h & 0xffffffu) + 0.5f) * (1.0f / 16777216.0f);
  const float r = sqrtf(-2.0f * logf(u1));
  float s, c;
  sincosf(6.28318530717958647692f * u2, &s, &c);
  const float z0 = r * c, z1 = r * s;
  if (BF16) {
    uint16_t* o = (uint16_t*)out;
    if (2 * j + 1 < n) *(uint32_t*)(o + 2 * j) = (uint32_t)to_bf16(z0) | ((uint32_t)to_bf16(z1) << 16);
    else o[2 * j] = to_bf16(z0);
  } else {
    float* o = (float*)out;
    o[2 * j] = z0;
    if (2 * j + 1 < n) o[2 * j + 1] = z1;
  }
}

}  // namespace

extern "C" {

// Fills out[0 .. n) (device memory, 4-byte aligned) with iid N(0,1) values of type `dtype`
// (0: fp32, 1: bf16) on `hip_stream`.  The values depend only on (seed, tensor_id, index, dtype).
// Returns 0, or 1 for a bad argument / refused launch.
int moda_synth_normal(void* out, unsigned long long n, unsigned long long seed, unsigned int tensor_id, int dtype,
                      void* hip_stream) {
  if (n == 0) return 0;
  if (!out || (dtype != 0 && dtype != 1) || ((uintptr_t)out & 3u)) return 1;
  const unsigned long long n_pairs = (n + 1) / 2;
  const unsigned long long blocks = (n_pairs + 255) / 256;
  if (blocks > 0x7fffffffull) return 1;
  const unsigned long long key = seed * 0x100000001b3ull + tensor_id;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (dtype == 1)
    hipLaunchKernelGGL(moda_synth_normal_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, out, n_pairs, n, key);
  else
    hipLaunchKernelGGL(moda_synth_normal_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, out, n_pairs, n, key);
  return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // extern "C"
