// MoDA attention forward, fp32 inputs, fp32 arithmetic on the vector ALUs.
//
// Accuracy path (max abs error 1e-5 against an fp64 evaluation is the target),
// not a throughput path: one wave per query.  Keys are walked 64 at a time, one
// key per lane: the lane computes the full dot product with fused multiply-adds
// in channel order, the wave agrees on the running max, and the value rows are
// accumulated with lane = channel.  The sequence keys and then the depth slots
// of the query's own position feed the SAME running max / normaliser / output
// (Algorithm 1), with one division at the end.
#include "moda_launch.h"

namespace moda {

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

template <int D>
struct F32State {
  float m, l;
  float o[D / 64];
};

// Fold `count` keys/values (rows of D floats, `stride` floats apart) into the state.
template <int D>
__device__ __forceinline__ void fold_keys(F32State<D>& st, const float* qs, const float* Kp,
                                          const float* Vp, int count, size_t stride, float scale,
                                          int lane) {
  for (int c0 = 0; c0 < count; c0 += 64) {
    const int j = c0 + lane;
    float s = -INFINITY;
    if (j < count) {
      const float4* kr = (const float4*)(Kp + (size_t)j * stride);
      float a = 0.f;
#pragma unroll 4
      for (int k = 0; k < D / 4; ++k) {
        float4 kv = kr[k];
        a = fmaf(qs[4 * k], kv.x, a);
        a = fmaf(qs[4 * k + 1], kv.y, a);
        a = fmaf(qs[4 * k + 2], kv.z, a);
        a = fmaf(qs[4 * k + 3], kv.w, a);
      }
      s = a * scale;
    }
    const float m_new = fmaxf(st.m, wave_max(s));
    const float alpha = expf(st.m - m_new);  // exp(-inf) = 0 on the first chunk
    const float pj = (j < count) ? expf(s - m_new) : 0.f;
    st.l = st.l * alpha + wave_sum(pj);
    st.m = m_new;
#pragma unroll
    for (int i = 0; i < D / 64; ++i) st.o[i] *= alpha;
    const int n = min(64, count - c0);
    for (int jj = 0; jj < n; ++jj) {
      const float pw = __shfl(pj, jj, 64);
      const float* vr = Vp + (size_t)(c0 + jj) * stride;
#pragma unroll
      for (int i = 0; i < D / 64; ++i) st.o[i] = fmaf(pw, vr[lane + 64 * i], st.o[i]);
    }
  }
}

template <int D>
__global__ __launch_bounds__(256) void moda_fwd_f32_kernel(FwdParams p) {
  __shared__ float qsm[4][D];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const long long row = (long long)blockIdx.x * 4 + wave;  // flat (b, h, t)
  const long long total = (long long)p.B * p.Hq * p.T;
  if (row >= total) return;  // whole wave leaves together; no block barrier is used below
  const int t = (int)(row % p.T);
  const int bh = (int)(row / p.T);
  const int b = bh / p.Hq;
  const int h = bh - b * p.Hq;
  const int g = h / (p.Hq / p.Hk);
  const size_t kvh = (size_t)(b * p.Hk + g);

  const float* q = (const float*)p.Q + (size_t)row * D;
  float* qs = qsm[wave];
#pragma unroll
  for (int i = 0; i < D / 64; ++i) qs[lane + 64 * i] = q[lane + 64 * i];
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  F32State<D> st;
  st.m = -INFINITY;
  st.l = 0.f;
#pragma unroll
  for (int i = 0; i < D / 64; ++i) st.o[i] = 0.f;

  const float* Ks = (const float*)p.Kseq + kvh * p.T * D;
  const float* Vs = (const float*)p.Vseq + kvh * p.T * D;
  fold_keys<D>(st, qs, Ks, Vs, p.causal ? t + 1 : p.T, D, p.scale, lane);
  if (p.depth_count > 0) {
    const size_t doff = (kvh * p.T + t) * (size_t)p.depth_alloc * D;
    fold_keys<D>(st, qs, (const float*)p.Kdepth + doff, (const float*)p.Vdepth + doff,
                 p.depth_count, D, p.scale, lane);
  }
  float* o = (float*)p.O + (size_t)row * D;
#pragma unroll
  for (int i = 0; i < D / 64; ++i) o[lane + 64 * i] = st.o[i] / st.l;
  if (lane == 0) p.LSE[row] = st.m + logf(st.l);
}

}  // namespace moda

namespace moda {

hipError_t launch_fwd_f32(const FwdParams& p, int d, hipStream_t stream) {
  const long long rows = (long long)p.B * p.Hq * p.T;
  const long long blocks = (rows + 3) / 4;
  if (!grid_ok(blocks)) return kGridTooLarge;
  dim3 grid((unsigned)blocks), block(256);
  if (d == 128) return launch_kernel(moda_fwd_f32_kernel<128>, grid, block, stream, p);
  if (d == 64) return launch_kernel(moda_fwd_f32_kernel<64>, grid, block, stream, p);
  return hipErrorInvalidValue;
}

}  // namespace moda
