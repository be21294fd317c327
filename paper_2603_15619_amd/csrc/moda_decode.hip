// MoDA attention for ONE new token per sequence (decoding; paper Table 1, "Decoding" rows).
// The new token's query attends the T positions of the sequence K/V cache (its own K/V
// included) and the depth slots of its own position, under one softmax (section 2.2); the
// depth cache of a decoding step is therefore only [B, Hk, depth_alloc, d].
//
// The call is bound by reading the sequence cache once (2 * B * Hk * T * d elements), so the
// keys are split over workgroups (one workgroup = one (batch, key/value head, slice of the
// sequence), all G query heads of the group together, so the slice is read once):
//   partial: per slice and head the running (max, normaliser, weighted value sum) in fp32,
//            written to the workspace;
//   merge  : per (batch, query head): folds the slices and the depth slots into one softmax,
//            normalises, stores O and LSE.
// Vector ALUs only (one query row per head: no matrix shape to speak of); a lane owns 8
// channels, d/8 lanes a key row, 64 / (d/8) key rows per wave instruction.
#include <atomic>

#include "moda_launch.h"

namespace moda {

constexpr int kDecWaves = 4;

// Scratch of the entry point that allocates nothing (moda_attn_decode_noalloc): the partial
// results of the slices, which the caller's workspace holds otherwise.  One copy per GPU, held
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress:
// kernels get the device address that call returns, never the name.
constexpr size_t kDecodeScratchBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kDecodeScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_addr[kMaxDevices];  // device address of `scratch`, per device (0: not looked up yet)

size_t decode_static_scratch_bytes() { return kDecodeScratchBytes; }

// Device address of `scratch` on the CURRENT device: looked up once per device (on the first
// call made with that device current), then served from the table.
hipError_t decode_static_scratch(void** addr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_addr[dev].store(p, std::memory_order_release);  // (two threads racing here store the same address)
  }
  *addr = p;
  return hipSuccess;
}

struct DecodeParams {
  const void* Q;       // [B, Hq, d]
  const void* Kseq;    // [B, Hk, T_alloc, d]
  const void* Vseq;
  const void* Kdepth;  // [B, Hk, depth_alloc, d]
  const void* Vdepth;
  void* O;             // [B, Hq, d]
  float* LSE;          // [B, Hq]
  float* ws;           // [B, Hq, n_split, d + 2]
  int B, Hq, Hk, T, T_alloc;
  int depth_alloc, depth_count;
  int n_split, keys_per_split;
  float scale, scale_log2;
};

template <int D, int GT>
__global__ __launch_bounds__(kDecWaves * 64) void moda_decode_partial_kernel(DecodeParams p) {
  constexpr int LPR = D / 8, RPS = 64 / LPR, RB = D * 2;
  __shared__ float red[kDecWaves][RPS][GT][D + 2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rg = lane / LPR, l16 = lane % LPR;
  const int G = p.Hq / p.Hk;
  const int n_gc = (G + GT - 1) / GT;  // head chunks per group
  int id = blockIdx.x;
  const int split = id % p.n_split;
  id /= p.n_split;
  const int gc = id % n_gc;
  const int bg = id / n_gc;  // (batch, key/value head)
  const int b = bg / p.Hk, g = bg - b * p.Hk;
  const int h0 = g * G + gc * GT;  // first query head of this chunk
  const float c2 = p.scale_log2;

  u32x4 q[GT];
  float m[GT], l[GT], o[GT][8];
#pragma unroll
  for (int j = 0; j < GT; ++j) {
    const int h = min(h0 + j, g * G + G - 1);  // heads past the group repeat the last one; never stored
    q[j] = *(const u32x4*)((const char*)p.Q + ((size_t)b * p.Hq + h) * RB + l16 * 16);
    m[j] = -INFINITY;
    l[j] = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) o[j][k] = 0.f;
  }
  const int k_begin = split * p.keys_per_split;
  const int k_end = min(p.T, k_begin + p.keys_per_split);
  const char* Kb = (const char*)p.Kseq + (size_t)bg * p.T_alloc * RB + l16 * 16;
  const char* Vb = (const char*)p.Vseq + (size_t)bg * p.T_alloc * RB + l16 * 16;

  // this lane's keys: k_begin + (wave * RPS + rg) + i * (kDecWaves * RPS), kU at a time with the
  // next kU in flight; the running max is raised (and the state rescaled) once per kU keys
  constexpr int STEP = kDecWaves * RPS;
  constexpr int kU = 4;
  const int key0 = k_begin + wave * RPS + rg;
  auto load = [&](const char* base, int kk) {
    return __builtin_nontemporal_load((const u32x4*)(base + (size_t)min(kk, p.T - 1) * RB));
  };
  u32x4 kn[kU], vn[kU];
#pragma unroll
  for (int u = 0; u < kU; ++u) {
    kn[u] = load(Kb, key0 + u * STEP);
    vn[u] = load(Vb, key0 + u * STEP);
  }
  for (int base = k_begin; base < k_end; base += kU * STEP) {  // uniform trip count over the workgroup
    const int key = key0 + (base - k_begin);
    u32x4 kv[kU], vv[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      kv[u] = kn[u];
      vv[u] = vn[u];
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      kn[u] = load(Kb, key + (kU + u) * STEP);
      vn[u] = load(Vb, key + (kU + u) * STEP);
    }
#pragma unroll
    for (int j = 0; j < GT; ++j) {
      float sc[kU];
      float mn = m[j];
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        float a = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) a = dot2_bf16(q[j][k], kv[u][k], a);
        a = group_sum<LPR>(a);
        sc[u] = key + u * STEP < k_end ? a : -INFINITY;
        mn = fmaxf(mn, sc[u]);
      }
      // (mn is -inf only while every key so far was past the slice: then nothing is added)
      const bool none = mn == -INFINITY;
      const float al = none ? 0.f : fast_exp2((m[j] - mn) * c2);
      m[j] = mn;
      l[j] *= al;
#pragma unroll
      for (int k = 0; k < 8; ++k) o[j][k] *= al;
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const float pw = none ? 0.f : fast_exp2((sc[u] - mn) * c2);
        l[j] += pw;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          o[j][2 * k] += pw * bf16_lo(vv[u][k]);
          o[j][2 * k + 1] += pw * bf16_hi(vv[u][k]);
        }
      }
    }
  }

  // ---- combine the (kDecWaves * RPS) row groups of the workgroup, per head
#pragma unroll
  for (int j = 0; j < GT; ++j) {
#pragma unroll
    for (int k = 0; k < 8; ++k) red[wave][rg][j][l16 * 8 + k] = o[j][k];
    if (l16 == 0) {
      red[wave][rg][j][D] = m[j];
      red[wave][rg][j][D + 1] = l[j];
    }
  }
  __syncthreads();
  // thread t < GT * D: head j = t / D, channel t % D
  for (int t = tid; t < GT * D; t += kDecWaves * 64) {
    const int j = t / D, ch = t % D;
    if (h0 + j >= g * G + G) continue;
    float mm = -INFINITY;
    for (int w = 0; w < kDecWaves; ++w)
      for (int r = 0; r < RPS; ++r) mm = fmaxf(mm, red[w][r][j][D]);
    float ll = 0.f, oo = 0.f;
    for (int w = 0; w < kDecWaves; ++w)
      for (int r = 0; r < RPS; ++r) {
        const float mi = red[w][r][j][D];
        const float f = mi == -INFINITY ? 0.f : fast_exp2((mi - mm) * c2);
        ll += f * red[w][r][j][D + 1];
        oo += f * red[w][r][j][ch];
      }
    float* dst = p.ws + (((size_t)b * p.Hq + h0 + j) * p.n_split + split) * (D + 2);
    dst[ch] = oo;
    if (ch == 0) {
      dst[D] = mm;
      dst[D + 1] = ll;
    }
  }
}

// One workgroup of D threads per (batch, query head): thread = channel.
template <int D>
__global__ __launch_bounds__(D) void moda_decode_merge_kernel(DecodeParams p) {
  __shared__ float sc_depth[64];
  __shared__ float qs[D];
  const int ch = threadIdx.x;
  const int bh = blockIdx.x;
  const int b = bh / p.Hq, h = bh - b * p.Hq;
  const int g = h / (p.Hq / p.Hk);
  const float c2 = p.scale_log2;
  const __bf16* Q = (const __bf16*)p.Q + (size_t)bh * D;
  qs[ch] = (float)Q[ch];
  __syncthreads();

  // slices of the sequence
  const float* ws = p.ws + (size_t)bh * p.n_split * (D + 2);
  float mm = -INFINITY;
  for (int s = 0; s < p.n_split; ++s) mm = fmaxf(mm, ws[s * (D + 2) + D]);
  // depth slots of the new token's position, 64 at a time: scores by the first threads
  const __bf16* Kd = (const __bf16*)p.Kdepth + (size_t)(b * p.Hk + g) * p.depth_alloc * D;
  const __bf16* Vd = (const __bf16*)p.Vdepth + (size_t)(b * p.Hk + g) * p.depth_alloc * D;
  float ll = 0.f, oo = 0.f, mref = mm;
  // pass 1 over the depth slots: maximum
  for (int i0 = 0; i0 < p.depth_count; i0 += 64) {
    const int n = min(64, p.depth_count - i0);
    __syncthreads();
    if (ch < n) {
      float a = 0.f;
      for (int k = 0; k < D; ++k) a += qs[k] * (float)Kd[(size_t)(i0 + ch) * D + k];
      sc_depth[ch] = a;
    }
    __syncthreads();
    for (int i = 0; i < n; ++i) mref = fmaxf(mref, sc_depth[i]);
  }
  for (int s = 0; s < p.n_split; ++s) {
    const float mi = ws[s * (D + 2) + D];
    const float f = mi == -INFINITY ? 0.f : fast_exp2((mi - mref) * c2);
    ll += f * ws[s * (D + 2) + D + 1];
    oo += f * ws[s * (D + 2) + ch];
  }
  // pass 2: weights and values
  for (int i0 = 0; i0 < p.depth_count; i0 += 64) {
    const int n = min(64, p.depth_count - i0);
    __syncthreads();
    if (ch < n) {
      float a = 0.f;
      for (int k = 0; k < D; ++k) a += qs[k] * (float)Kd[(size_t)(i0 + ch) * D + k];
      sc_depth[ch] = a;
    }
    __syncthreads();
    for (int i = 0; i < n; ++i) {
      const float pw = fast_exp2((sc_depth[i] - mref) * c2);
      ll += pw;
      oo += pw * (float)Vd[(size_t)(i0 + i) * D + ch];
    }
  }
  ((__bf16*)p.O)[(size_t)bh * D + ch] = (__bf16)(oo / ll);
  if (ch == 0) p.LSE[bh] = mref * p.scale + __logf(ll);
}

int decode_splits(int B, int Hk, int T) {
  // enough workgroups to fill 256 compute units a few times over, slices of at least 256 keys
  const int want = (2048 + B * Hk - 1) / (B * Hk);
  const int most = (T + 255) / 256;
  int s = want < most ? want : most;
  return s < 1 ? 1 : s;
}

size_t decode_workspace_bytes(int B, int Hq, int Hk, int T, int d) {
  return (size_t)B * Hq * decode_splits(B, Hk, T) * (d + 2) * sizeof(float);
}

template <int D>
static hipError_t launch_decode_d(DecodeParams p, hipStream_t stream) {
  const int G = p.Hq / p.Hk;
  const int gt = G >= 8 ? 8 : G >= 4 ? 4 : G >= 2 ? 2 : 1;
  const int n_gc = (G + gt - 1) / gt;
  const long long blocks = (long long)p.B * p.Hk * n_gc * p.n_split;
  if (!grid_ok(blocks) || !grid_ok((long long)p.B * p.Hq)) return kGridTooLarge;
  dim3 grid((unsigned)blocks), block(kDecWaves * 64);
  hipError_t e;
  if (gt == 8) e = launch_kernel(moda_decode_partial_kernel<D, 8>, grid, block, stream, p);
  else if (gt == 4) e = launch_kernel(moda_decode_partial_kernel<D, 4>, grid, block, stream, p);
  else if (gt == 2) e = launch_kernel(moda_decode_partial_kernel<D, 2>, grid, block, stream, p);
  else e = launch_kernel(moda_decode_partial_kernel<D, 1>, grid, block, stream, p);
  if (e != hipSuccess) return e;
  return launch_kernel(moda_decode_merge_kernel<D>, dim3((unsigned)(p.B * p.Hq)), dim3(D), stream, p);
}

hipError_t launch_decode_bf16(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                              const void* Vdepth, void* O, float* LSE, float* ws, int B, int Hq, int Hk, int T,
                              int T_alloc, int d, int depth_alloc, int depth_count, float scale,
                              hipStream_t stream) {
  DecodeParams p;
  p.Q = Q; p.Kseq = Kseq; p.Vseq = Vseq; p.Kdepth = Kdepth; p.Vdepth = Vdepth;
  p.O = O; p.LSE = LSE; p.ws = ws;
  p.B = B; p.Hq = Hq; p.Hk = Hk; p.T = T; p.T_alloc = T_alloc;
  p.depth_alloc = depth_alloc; p.depth_count = depth_count;
  p.n_split = decode_splits(B, Hk, T);
  // slices are multiples of the key rows a workgroup takes per step (16 or 32)
  const int step = kDecWaves * (64 / (d / 8));
  p.keys_per_split = ((T + p.n_split - 1) / p.n_split + step - 1) / step * step;
  p.scale = scale;
  p.scale_log2 = scale * 1.4426950408889634f;
  if (d == 128) return launch_decode_d<128>(p, stream);
  if (d == 64) return launch_decode_d<64>(p, stream);
  return hipErrorInvalidValue;
}

}  // namespace moda
