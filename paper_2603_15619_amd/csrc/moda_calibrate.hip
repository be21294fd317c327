// Calibration kernel: what the matrix pipe alone sustains on this chip, for the data it is
// given.  Nothing but v_mfma_f32_32x32x16_bf16 in the loop: four independent accumulators per
// wave, operands loaded once from `operands` (so the caller chooses their values: the sustained
// rate depends on them, the chip lowers its clock under the power that random operands draw),
// eight waves per workgroup (two per SIMD), as the attention kernels run.  Timed by the caller.
#include "moda_launch.h"

namespace moda {

constexpr int kCalibThreads = 512;
constexpr int kCalibAcc = 4;

__global__ __launch_bounds__(kCalibThreads) void moda_calibrate_mfma_kernel(const bf16x8* operands, float* sink,
                                                                          int iters) {
  bf16x8 a[kCalibAcc], b[kCalibAcc];
#pragma unroll
  for (int i = 0; i < kCalibAcc; ++i) {
    a[i] = operands[i * kCalibThreads + threadIdx.x];
    b[i] = operands[(kCalibAcc + i) * kCalibThreads + threadIdx.x];
  }
  f32x16 c[kCalibAcc] = {};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kCalibAcc; ++i) c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], c[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kCalibAcc; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) s += c[i][j];
  sink[(size_t)blockIdx.x * kCalibThreads + threadIdx.x] = s;
}

size_t calibrate_operand_bytes() { return (size_t)2 * kCalibAcc * kCalibThreads * sizeof(bf16x8); }
size_t calibrate_sink_bytes(int workgroups) { return (size_t)workgroups * kCalibThreads * sizeof(float); }
double calibrate_flops(int workgroups, int iters) {
  return 2.0 * 32 * 32 * 16 * kCalibAcc * (double)iters * (kCalibThreads / 64) * workgroups;
}

hipError_t launch_calibrate_mfma(const void* operands, float* sink, int workgroups, int iters, hipStream_t stream) {
  if (!grid_ok(workgroups) || iters < 0) return kGridTooLarge;
  return launch_kernel(moda_calibrate_mfma_kernel, dim3((unsigned)workgroups), dim3(kCalibThreads), stream,
                       (const bf16x8*)operands, sink, iters);
}

}  // namespace moda
