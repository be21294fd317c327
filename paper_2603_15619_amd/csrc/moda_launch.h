// Host-side launchers, one per kernel family; implemented next to the kernels.
#pragma once
#include "moda_common.h"

namespace moda {

// Enqueues `kernel` and returns THIS launch's status (hipLaunchKernel's own return value; the
// thread's sticky "last error", which earlier work of the caller may have set, is not read).
template <class... Params, class... Args>
inline hipError_t launch_kernel(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream, Args... args) {
  static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
  return [&](Params... a) {
    void* argv[] = {(void*)&a...};
    return hipLaunchKernel((const void*)kernel, grid, block, argv, 0, stream);
  }(args...);
}
// A grid that does not fit a launch: reported before anything is enqueued (the C ABI turns it
// into MODA_ERR_UNSUPPORTED).
constexpr hipError_t kGridTooLarge = hipErrorInvalidConfiguration;
inline bool grid_ok(long long blocks) { return blocks > 0 && blocks <= 0x7fffffffLL; }

// bf16 forward kernel: `waves` (8 or 4) waves per workgroup, 32 queries each; p.n_qtiles
// must be the number of such tiles in p.T.
int fwd_bf16_tile_rows(int waves);
hipError_t launch_fwd_bf16(const FwdParams& p, int d, int waves, hipStream_t stream);
hipError_t launch_fwd_f32(const FwdParams& p, int d, hipStream_t stream);

// Backward (bf16, Hq / Hk <= bwd_bf16_max_group()): delta, [depth slots of grouped queries,]
// dK/dV and dQ(/depth) kernels on `stream`.
int bwd_bf16_max_group();
int bwd_bf16_kernels(const BwdParams& p);  // kernels one call enqueues
size_t bwd_bf16_workspace_bytes(const BwdParams& p, int d);
hipError_t launch_bwd_bf16(const BwdParams& p, int d, hipStream_t stream);

// Depth-stream write step: rows of K / V [rows, row_bytes] into slot `slot` of
// [rows, depth_alloc, row_bytes].
hipError_t launch_depth_append(const void* K, const void* V, void* Kdepth, void* Vdepth, long long rows,
                               int row_bytes, int depth_alloc, int slot, hipStream_t stream);

// Decoding step (one new token per sequence), bf16: partial kernel over slices of the sequence
// cache + merge kernel; `ws` holds decode_workspace_bytes(...) bytes.
size_t decode_workspace_bytes(int B, int Hq, int Hk, int T, int d);
// The library's own scratch for the decoding step (a file-scope device array, one per GPU): its
// size, and its device address on the current device.
size_t decode_static_scratch_bytes();
hipError_t decode_static_scratch(void** addr);
hipError_t launch_decode_bf16(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                              const void* Vdepth, void* O, float* LSE, float* ws, int B, int Hq, int Hk, int T,
                              int T_alloc, int d, int depth_alloc, int depth_count, float scale,
                              hipStream_t stream);

// Matrix-pipe calibration kernel (moda_calibrate.hip).
size_t calibrate_operand_bytes();
size_t calibrate_sink_bytes(int workgroups);
double calibrate_flops(int workgroups, int iters);
hipError_t launch_calibrate_mfma(const void* operands, float* sink, int workgroups, int iters, hipStream_t stream);

}  // namespace moda
